"""Thin ctypes binding over libq8.so (the C ABI declared in include/q8.h).

Argument marshalling only: every step of the quantized FC layer runs in the HIP
kernels behind the library.  PyTorch supplies device memory and the stream.
Importing this module fails loudly when the library has not been built
(`python -m paper_1910_06188_amd.build`); there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libq8.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first (python -m paper_1910_06188_amd.build). "
        "There is no fallback path.")

_lib = C.CDLL(LIB_PATH)

OK = 0
EPI_GELU, EPI_ABSMAX, EPI_REQUANT = 1, 2, 4
MAX_K = 131071
STATIC_MAX_CODES = 64 << 20
SCAL_WORK = 2050
AMAX_SLOTS = 2048

_vp, _i64, _i32, _u32 = C.c_void_p, C.c_int64, C.c_int, C.c_uint32

_lib.q8_absmax.argtypes = [_vp, _i64, _vp, _vp, _vp]
_lib.q8_scale_from_amax.argtypes = [_vp, _vp, _vp]
_lib.q8_quantize.argtypes = [_vp, _i64, _vp, _vp, _vp]
_lib.q8_quantize_amax.argtypes = [_vp, _i64, _vp, _i32, _vp, _vp, _vp, _vp]
_lib.q8_linear.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _u32, _vp]
_lib.q8_linear_residual.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _u32, _vp]
_lib.q8_linear_residual.restype = C.c_int
_lib.q8_linear_f32.argtypes = [_vp, _vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _vp]
_lib.q8_embedding.argtypes = [_vp, _vp, _i64, _i64, _vp, _i64, _vp, _i32, _vp, _vp]
_lib.q8_embedding_sum3.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _vp]
_f32 = C.c_float
_lib.q8_fake_quantize.argtypes = [_vp, _i64, _vp, _vp, _vp]
_lib.q8_ema_update.argtypes = [_vp, _i32, _f32, _vp, _vp, _vp, _vp]
_lib.q8_fake_quantize_ema.argtypes = [_vp, _i64, _f32, _vp, _vp, _vp, _vp]
_lib.q8_ste_backward.argtypes = [_vp, _i64, _vp, _vp]
_lib.q8_layernorm_absmax.argtypes = [_vp, _vp, _vp, _vp, _f32, _i64, _i64, _vp, _vp, _vp, _vp, _vp]
_lib.q8_embedding_sum3_layernorm.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _f32,
                                             _vp, _vp, _vp, _vp, _vp, _vp]
_lib.q8_attention.argtypes = [_vp, _i64, _i64, _i32, _i32, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
_lib.q8_linear_f32_static.argtypes = [_vp, _vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _u32, _vp]
_lib.q8_linear_f32_static.restype = C.c_int
_lib.q8_quantize_dynamic.argtypes = [_vp, _i64, _vp, _vp, _vp, _vp]
_lib.q8_quantize_dynamic.restype = C.c_int
_lib.q8_debug_mfma_rate.argtypes = [_vp, _i32, _i32, _vp, _vp]
_lib.q8_debug_mfma_rate.restype = C.c_int
_lib.q8_debug_stream_copy.argtypes = [_vp, _vp, _i64, _vp]
_lib.q8_debug_stream_copy.restype = C.c_int
_lib.q8_debug_loop_probe.argtypes = [_i32, _vp, _vp, _i32, _vp, _vp]
_lib.q8_debug_loop_probe.restype = C.c_int
_lib.q8_linear_f32_slots.argtypes = [_vp, _vp, _i32, _vp, _vp, _vp, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _u32, _vp]
for _f in ("q8_linear_f32_slots", "q8_attention", "q8_layernorm_absmax", "q8_embedding_sum3_layernorm", "q8_fake_quantize", "q8_ema_update", "q8_fake_quantize_ema", "q8_ste_backward", "q8_absmax", "q8_scale_from_amax", "q8_quantize", "q8_quantize_amax", "q8_linear", "q8_linear_f32", "q8_embedding",
           "q8_embedding_sum3"):
    getattr(_lib, _f).restype = C.c_int
_lib.q8_version.restype = C.c_char_p
_lib.q8_status_str.restype = C.c_char_p
_lib.q8_status_str.argtypes = [C.c_int]
_lib.q8_debug_set_gemm_variant.argtypes = [C.c_int]
_lib.q8_debug_set_gemm_variant.restype = None
_lib.q8_debug_set_quantize_one_pass.argtypes = [C.c_int, _u32]
_lib.q8_debug_set_quantize_one_pass.restype = None


class Q8Error(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {_lib.q8_status_str(code).decode()} (status {code})")
        self.code = code


def _ck(code: int, where: str) -> None:
    if code != OK:
        raise Q8Error(code, where)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("q8 takes device tensors")
    if not t.is_contiguous():
        raise ValueError("q8 takes contiguous tensors")
    return t.data_ptr()


# The current stream's raw handle without building a torch.cuda.Stream object for it (2.7 us per call, about
# as much as the launch itself); the public accessor is the fallback.
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream=None):
    if stream is not None:
        return stream.cuda_stream
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def version() -> str:
    return _lib.q8_version().decode()


def status_str(code: int) -> str:
    return _lib.q8_status_str(code).decode()


def set_gemm_variant(v: int) -> None:
    _lib.q8_debug_set_gemm_variant(int(v))


def set_quantize_one_pass(enabled: bool = True, barrier_polls: int = 64) -> None:
    """Tuning hook of the dynamic quantizer's one-pass kernel (off: two passes; barrier_polls 0: never wait)."""
    _lib.q8_debug_set_quantize_one_pass(1 if enabled else 0, int(barrier_polls))


def q8_absmax(x, amax_out, scale_out=None, stream=None) -> None:
    """amax_out[0] = max|x|, scale_out[0] = 127/amax (Eq. 3)."""
    _ck(_lib.q8_absmax(_ptr(x), x.numel(), _ptr(amax_out), _ptr(scale_out), _stream(stream)), "q8_absmax")


def q8_scale_from_amax(amax, scale_out, stream=None) -> None:
    _ck(_lib.q8_scale_from_amax(_ptr(amax), _ptr(scale_out), _stream(stream)), "q8_scale_from_amax")


def q8_quantize(x, scale, q, stream=None) -> None:
    """q = Clamp(round(x * scale), -127, 127) (Eq. 1)."""
    if q.numel() != x.numel():
        raise ValueError("q8_quantize: q and x differ in size")
    _ck(_lib.q8_quantize(_ptr(x), x.numel(), _ptr(scale), _ptr(q), _stream(stream)), "q8_quantize")


def q8_quantize_amax(x, amax, scale_out, q, amax_out=None, stream=None) -> None:
    """S = 127 / max(amax[:]) (Eq. 3), then q = Quantize(x | S, 127) (Eq. 1), one launch."""
    if q.numel() != x.numel():
        raise ValueError("q8_quantize_amax: q and x differ in size")
    _ck(_lib.q8_quantize_amax(_ptr(x), x.numel(), _ptr(amax), amax.numel(), _ptr(amax_out), _ptr(scale_out), _ptr(q),
                              _stream(stream)), "q8_quantize_amax")


def q8_quantize_dynamic(x, q, scal_work, zero_slot=None, stream=None) -> None:
    """Dynamic quantizer (Section 4.1): scal_work[0] = max|x|, scal_work[1] = S = 127/max, q = Quantize(x | S, 127)."""
    if q.numel() != x.numel() or scal_work.numel() < SCAL_WORK:
        raise ValueError("q8_quantize_dynamic: shape mismatch")
    _ck(_lib.q8_quantize_dynamic(_ptr(x), x.numel(), _ptr(q), _ptr(scal_work), _ptr(zero_slot), _stream(stream)),
        "q8_quantize_dynamic")


def debug_mfma_rate(operands, iters, workgroups, sink, stream=None) -> float:
    """Launches the register-resident i8 MFMA loop; returns the int8 operations it performs."""
    if operands.numel() < 65536:
        raise ValueError("debug_mfma_rate: operands holds 65536 int8 values")
    _ck(_lib.q8_debug_mfma_rate(_ptr(operands), int(iters), int(workgroups), _ptr(sink), _stream(stream)), "q8_debug_mfma_rate")
    return 2.0 * 32 * 32 * 32 * 8 * iters * 8 * workgroups


def debug_stream_copy(src, dst, stream=None) -> None:
    """dst = src with 16-byte accesses (src None: fill)."""
    nbytes = dst.numel() * dst.element_size()
    _ck(_lib.q8_debug_stream_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "q8_debug_stream_copy")


def debug_loop_probe(what, operand_window, store_window, stages, sink, stream=None) -> None:
    """One stage of a GEMM main loop piece by piece (see include/q8.h); 256 workgroups x `stages` stages."""
    if operand_window.numel() * operand_window.element_size() < (4 << 20) or store_window.numel() * store_window.element_size() < (32 << 20):
        raise ValueError("debug_loop_probe: windows of 4 MiB and 32 MiB")
    _ck(_lib.q8_debug_loop_probe(int(what), _ptr(operand_window), _ptr(store_window), int(stages), _ptr(sink), _stream(stream)),
        "q8_debug_loop_probe")


def q8_linear(xq, wq, bias, sx, sw, y, n_groups=1, acc_out=None, out_amax=None, next_scale=None, flags=0,
              stream=None) -> None:
    """y = dequant(xq wq^T + quantized bias) (Section 3), optional fused epilogue stages."""
    M, K = xq.shape
    N, K2 = wq.shape
    if K != K2 or y.numel() != M * N or (acc_out is not None and acc_out.numel() != M * N):
        raise ValueError("q8_linear: shape mismatch")
    if sw.numel() != n_groups or (bias is not None and bias.numel() != N):
        raise ValueError("q8_linear: scale/bias size mismatch")
    _ck(_lib.q8_linear(_ptr(xq), _ptr(wq), _ptr(bias), _ptr(sx), _ptr(sw), n_groups, M, N, K, _ptr(y),
                       _ptr(acc_out), _ptr(out_amax), _ptr(next_scale), flags, _stream(stream)), "q8_linear")


def q8_linear_residual(xq, wq, bias, sx, sw, residual, y, n_groups=1, acc_out=None, out_amax=None, flags=0,
                       stream=None) -> None:
    """y = dequant(xq wq^T + quantized bias) + residual: the FC layer with the encoder's residual addition fused."""
    M, K = xq.shape
    N, K2 = wq.shape
    if K != K2 or y.numel() != M * N or residual.numel() != M * N or (acc_out is not None and acc_out.numel() != M * N):
        raise ValueError("q8_linear_residual: shape mismatch")
    if sw.numel() != n_groups or (bias is not None and bias.numel() != N):
        raise ValueError("q8_linear_residual: scale/bias size mismatch")
    _ck(_lib.q8_linear_residual(_ptr(xq), _ptr(wq), _ptr(bias), _ptr(sx), _ptr(sw), n_groups, M, N, K, _ptr(residual),
                                _ptr(y), _ptr(acc_out), _ptr(out_amax), flags, _stream(stream)), "q8_linear_residual")


def q8_linear_f32(x, wq, bias, sw, xq_work, scal_work, y, n_groups=1, acc_out=None, out_amax=None, next_scale=None,
                  flags=0, stream=None) -> None:
    """Dynamic-quantization FC layer in one call: abs-max, quantize, GEMM, dequantize."""
    M, K = x.shape
    N, K2 = wq.shape
    if K != K2 or y.numel() != M * N or xq_work.numel() < M * K or scal_work.numel() < SCAL_WORK:
        raise ValueError("q8_linear_f32: shape mismatch")
    if sw.numel() != n_groups or (bias is not None and bias.numel() != N):
        raise ValueError("q8_linear_f32: scale/bias size mismatch")
    _ck(_lib.q8_linear_f32(_ptr(x), _ptr(wq), _ptr(bias), _ptr(sw), n_groups, M, N, K, _ptr(xq_work),
                           _ptr(scal_work), _ptr(y), _ptr(acc_out), _ptr(out_amax), _ptr(next_scale), flags,
                           _stream(stream)), "q8_linear_f32")


def q8_linear_f32_static(x, wq, bias, sw, y, n_groups=1, stats_out=None, out_amax=None, next_scale=None, flags=0,
                         stream=None) -> None:
    """q8_linear_f32 on the library's static scratch: no workspace arguments, nothing allocated."""
    M, K = x.shape
    N, K2 = wq.shape
    if K != K2 or y.numel() != M * N or (stats_out is not None and stats_out.numel() < 2):
        raise ValueError("q8_linear_f32_static: shape mismatch")
    if sw.numel() != n_groups or (bias is not None and bias.numel() != N):
        raise ValueError("q8_linear_f32_static: scale/bias size mismatch")
    _ck(_lib.q8_linear_f32_static(_ptr(x), _ptr(wq), _ptr(bias), _ptr(sw), n_groups, M, N, K, _ptr(y), _ptr(stats_out),
                                  _ptr(out_amax), _ptr(next_scale), flags, _stream(stream)), "q8_linear_f32_static")


def q8_linear_f32_slots(x, amax_slots, wq, bias, sw, xq_work, scal_work, y, n_groups=1, acc_out=None, out_amax=None,
                        next_scale=None, flags=0, stream=None) -> None:
    """Dynamic-quantization FC layer fed by abs-max slots its producer left: quantize (scale from the slots), GEMM."""
    M, K = x.shape
    N, K2 = wq.shape
    if K != K2 or y.numel() != M * N or xq_work.numel() < M * K or scal_work.numel() < 2 or amax_slots.numel() < 1:
        raise ValueError("q8_linear_f32_slots: shape mismatch")
    if sw.numel() != n_groups or (bias is not None and bias.numel() != N):
        raise ValueError("q8_linear_f32_slots: scale/bias size mismatch")
    _ck(_lib.q8_linear_f32_slots(_ptr(x), _ptr(amax_slots), amax_slots.numel(), _ptr(wq), _ptr(bias), _ptr(sw), n_groups,
                                 M, N, K, _ptr(xq_work), _ptr(scal_work), _ptr(y), _ptr(acc_out), _ptr(out_amax),
                                 _ptr(next_scale), flags, _stream(stream)), "q8_linear_f32_slots")


def q8_embedding(table, scale, ids, out, err_flag=None, stream=None) -> None:
    """out[t] = table[ids[t]] (int8 out) or table[ids[t]] / scale (fp32 out)."""
    V, H = table.shape
    T = ids.numel()
    if out.numel() != T * H:
        raise ValueError("q8_embedding: shape mismatch")
    out_is_int8 = 1 if out.dtype == torch.int8 else 0
    _ck(_lib.q8_embedding(_ptr(table), _ptr(scale), V, H, _ptr(ids), T, _ptr(out), out_is_int8, _ptr(err_flag),
                          _stream(stream)), "q8_embedding")


def q8_embedding_sum3(word, pos, typ, scales, wid, pid, tid, out, err_flag=None, stream=None) -> None:
    H = word.shape[1]
    T = wid.numel()
    if pos.shape[1] != H or typ.shape[1] != H or out.numel() != T * H or pid.numel() != T or tid.numel() != T:
        raise ValueError("q8_embedding_sum3: shape mismatch")
    _ck(_lib.q8_embedding_sum3(_ptr(word), word.shape[0], _ptr(pos), pos.shape[0], _ptr(typ), typ.shape[0],
                               _ptr(scales), H, _ptr(wid), _ptr(pid), _ptr(tid), T, _ptr(out), _ptr(err_flag),
                               _stream(stream)), "q8_embedding_sum3")


def q8_fake_quantize(x, scale, xq, stream=None) -> None:
    """xq = Quantize(x | S, 127) / S in fp32 (Section 2.2); xq may be x."""
    if xq.numel() != x.numel():
        raise ValueError("q8_fake_quantize: xq and x differ in size")
    _ck(_lib.q8_fake_quantize(_ptr(x), x.numel(), _ptr(scale), _ptr(xq), _stream(stream)), "q8_fake_quantize")


def q8_ema_update(amax, decay, state, amax_out=None, scale_out=None, stream=None) -> None:
    """One step of the moving average of max|x| under Eq. 4; state = [average, started]."""
    if state.numel() < 2:
        raise ValueError("q8_ema_update: state holds two floats")
    _ck(_lib.q8_ema_update(_ptr(amax), amax.numel(), float(decay), _ptr(state), _ptr(amax_out), _ptr(scale_out),
                           _stream(stream)), "q8_ema_update")


def q8_fake_quantize_ema(x, decay, state, scal_work, xq, stream=None) -> None:
    """abs-max, moving-average step, fake quantization with the updated scale, in one call."""
    if xq.numel() != x.numel() or state.numel() < 2 or scal_work.numel() < SCAL_WORK:
        raise ValueError("q8_fake_quantize_ema: shape mismatch")
    _ck(_lib.q8_fake_quantize_ema(_ptr(x), x.numel(), float(decay), _ptr(state), _ptr(scal_work), _ptr(xq),
                                  _stream(stream)), "q8_fake_quantize_ema")


def q8_ste_backward(grad_xq, grad_x, stream=None) -> None:
    """Eq. 5: grad_x = grad_xq."""
    if grad_x.numel() != grad_xq.numel():
        raise ValueError("q8_ste_backward: sizes differ")
    _ck(_lib.q8_ste_backward(_ptr(grad_xq), grad_xq.numel(), _ptr(grad_x), _stream(stream)), "q8_ste_backward")


def q8_layernorm_absmax(a, gamma, beta, y, eps=1e-12, residual=None, amax_slots=None, q_scale=None, q_out=None,
                        stream=None) -> None:
    """y = LayerNorm(a (+ residual)) * gamma + beta, plus abs-max slots of y for the next quantizer, or
    (stored scale) the int8 codes of y themselves."""
    M, H = a.shape
    if y.numel() != M * H or gamma.numel() != H or beta.numel() != H or (residual is not None and residual.numel() != M * H):
        raise ValueError("q8_layernorm_absmax: shape mismatch")
    if amax_slots is not None and amax_slots.numel() < AMAX_SLOTS:
        raise ValueError("q8_layernorm_absmax: amax_slots holds AMAX_SLOTS floats")
    if q_out is not None and q_out.numel() != M * H:
        raise ValueError("q8_layernorm_absmax: q_out and y differ in size")
    _ck(_lib.q8_layernorm_absmax(_ptr(a), _ptr(residual), _ptr(gamma), _ptr(beta), float(eps), M, H, _ptr(y),
                                 _ptr(amax_slots), _ptr(q_scale), _ptr(q_out), _stream(stream)), "q8_layernorm_absmax")


def q8_embedding_sum3_layernorm(word, pos, typ, scales, wid, pid, tid, gamma, beta, y, eps=1e-12, amax_slots=None,
                                q_scale=None, q_out=None, err_flag=None, stream=None) -> None:
    """Three-table int8 lookup, sum, LayerNorm and abs-max slots in one pass."""
    H = word.shape[1]
    T = wid.numel()
    if pos.shape[1] != H or typ.shape[1] != H or y.numel() != T * H or pid.numel() != T or tid.numel() != T:
        raise ValueError("q8_embedding_sum3_layernorm: shape mismatch")
    if gamma.numel() != H or beta.numel() != H or (amax_slots is not None and amax_slots.numel() < AMAX_SLOTS):
        raise ValueError("q8_embedding_sum3_layernorm: parameter size mismatch")
    _ck(_lib.q8_embedding_sum3_layernorm(_ptr(word), word.shape[0], _ptr(pos), pos.shape[0], _ptr(typ), typ.shape[0],
                                         _ptr(scales), H, _ptr(wid), _ptr(pid), _ptr(tid), T, _ptr(gamma), _ptr(beta),
                                         float(eps), _ptr(y), _ptr(amax_slots), _ptr(q_scale), _ptr(q_out), _ptr(err_flag),
                                         _stream(stream)),
        "q8_embedding_sum3_layernorm")


def q8_attention(qkv, B, S, heads, d, ctx=None, mask=None, scale=None, amax_slots=None, q_scale=None, q_out=None,
                 stream=None) -> None:
    """ctx = softmax(scale * Q K^T + mask) V per head on the fused projection output qkv [B*S, 3*heads*d], plus
    abs-max slots of ctx for the next quantizer, or (stored scale) the int8 codes of ctx themselves."""
    if qkv.numel() != B * S * 3 * heads * d:
        raise ValueError("q8_attention: qkv does not hold B*S rows of 3*heads*d columns")
    if ctx is not None and ctx.numel() != B * S * heads * d:
        raise ValueError("q8_attention: ctx size mismatch")
    if q_out is not None and q_out.numel() != B * S * heads * d:
        raise ValueError("q8_attention: q_out size mismatch")
    if mask is not None and mask.numel() != B * S:
        raise ValueError("q8_attention: mask holds one value per (sequence, key)")
    if amax_slots is not None and amax_slots.numel() < AMAX_SLOTS:
        raise ValueError("q8_attention: amax_slots holds AMAX_SLOTS floats")
    if scale is None:
        scale = 1.0 / float(d) ** 0.5
    _ck(_lib.q8_attention(_ptr(qkv), B, S, heads, d, _ptr(mask), float(scale), _ptr(ctx), _ptr(amax_slots), _ptr(q_scale),
                          _ptr(q_out), _stream(stream)), "q8_attention")


def raw():
    """The ctypes library handle, for tests that call the C ABI with unusual arguments."""
    return _lib
