"""ctypes front end of the q8 CPU oracle -- TEST INFRASTRUCTURE ONLY.

Builds oracle/q8_oracle.c with gcc and exposes each step of the quantized
fully-connected layer (Q8BERT, Sections 2.1, 3 and 4.1) on NumPy arrays.  Nothing
in the product package imports this module; only tests, the smoke check and the
benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "q8_oracle.c")
_LIB = os.path.join(_HERE, "libq8_oracle.so")

OK, ERR_NONFINITE, ERR_OVERFLOW, ERR_INDEX, ERR_SHAPE = 0, 1, 2, 3, 4


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle {where}: error {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the C oracle (separately rounded fp32 ops, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def _check(code: int, where: str):
    if code != OK:
        raise OracleError(code, where)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def absmax(x) -> np.float32:
    x = _f32(x)
    out = C.c_float()
    _check(lib().q8o_absmax(_p(x, C.c_float), C.c_int64(x.size), C.byref(out)), "absmax")
    return np.float32(out.value)


def scale(amax) -> np.float32:
    out = C.c_float()
    _check(lib().q8o_scale(C.c_float(float(amax)), C.byref(out)), "scale")
    return np.float32(out.value)


def quantize(x, s) -> np.ndarray:
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.int8)
    _check(lib().q8o_quantize(_p(x, C.c_float), C.c_int64(x.size), C.c_float(float(s)), _p(q, C.c_int8)),
           "quantize")
    return q


def quantize_bias(b, n, sx, sw) -> np.ndarray:
    sw = np.atleast_1d(_f32(sw))
    bq = np.empty(n, dtype=np.int32)
    bp = None
    if b is not None:
        b = _f32(b)
        bp = _p(b, C.c_float)
    _check(lib().q8o_quantize_bias(bp, C.c_int64(n), C.c_float(float(sx)), _p(sw, C.c_float),
                                   C.c_int(sw.size), _p(bq, C.c_int32)), "quantize_bias")
    return bq


def gemm_i8(xq, wq, bq=None, threads: int = 1) -> np.ndarray:
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    if K != K2:
        raise OracleError(ERR_SHAPE, "gemm_i8")
    acc = np.empty((M, N), dtype=np.int32)
    bp = None
    if bq is not None:
        bq = np.ascontiguousarray(bq, dtype=np.int32)
        bp = _p(bq, C.c_int32)
    _check(lib().q8o_gemm_i8(_p(xq, C.c_int8), _p(wq, C.c_int8), bp, C.c_int64(M), C.c_int64(N),
                             C.c_int64(K), _p(acc, C.c_int32), C.c_int(threads)), "gemm_i8")
    return acc


def dequant(acc, sx, sw) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    sw = np.atleast_1d(_f32(sw))
    M, N = acc.shape
    y = np.empty((M, N), dtype=np.float32)
    _check(lib().q8o_dequant(_p(acc, C.c_int32), C.c_int64(M), C.c_int64(N), C.c_float(float(sx)),
                             _p(sw, C.c_float), C.c_int(sw.size), _p(y, C.c_float)), "dequant")
    return y


def gelu(v) -> np.ndarray:
    v = _f32(v)
    out = np.empty_like(v)
    lib().q8o_gelu(_p(v, C.c_float), C.c_int64(v.size), _p(out, C.c_float))
    return out


def embedding(table_q, s, ids, want_f32: bool = True):
    table_q = np.ascontiguousarray(table_q, dtype=np.int8)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    V, H = table_q.shape
    T = ids.size
    out_i8 = np.empty((T, H), dtype=np.int8)
    out_f = np.empty((T, H), dtype=np.float32) if want_f32 else None
    _check(lib().q8o_embedding(_p(table_q, C.c_int8), C.c_int64(V), C.c_int64(H), C.c_float(float(s)),
                               _p(ids, C.c_int32), C.c_int64(T), _p(out_i8, C.c_int8),
                               None if out_f is None else _p(out_f, C.c_float)), "embedding")
    return out_i8, out_f


def embedding_sum3(word_q, s_word, pos_q, s_pos, typ_q, s_typ, wid, pid, tid) -> np.ndarray:
    word_q = np.ascontiguousarray(word_q, dtype=np.int8)
    pos_q = np.ascontiguousarray(pos_q, dtype=np.int8)
    typ_q = np.ascontiguousarray(typ_q, dtype=np.int8)
    wid = np.ascontiguousarray(wid, dtype=np.int32)
    pid = np.ascontiguousarray(pid, dtype=np.int32)
    tid = np.ascontiguousarray(tid, dtype=np.int32)
    H = word_q.shape[1]
    T = wid.size
    out = np.empty((T, H), dtype=np.float32)
    _check(lib().q8o_embedding_sum3(
        _p(word_q, C.c_int8), C.c_int64(word_q.shape[0]), C.c_float(float(s_word)),
        _p(pos_q, C.c_int8), C.c_int64(pos_q.shape[0]), C.c_float(float(s_pos)),
        _p(typ_q, C.c_int8), C.c_int64(typ_q.shape[0]), C.c_float(float(s_typ)),
        C.c_int64(H), _p(wid, C.c_int32), _p(pid, C.c_int32), _p(tid, C.c_int32), C.c_int64(T),
        _p(out, C.c_float)), "embedding_sum3")
    return out



def fake_quantize(x, s) -> np.ndarray:
    """x^q = Quantize(x | S, 127) / S in fp32 (Section 2.2)."""
    x = _f32(x)
    y = np.empty(x.shape, dtype=np.float32)
    _check(lib().q8o_fake_quantize(_p(x, C.c_float), C.c_int64(x.size), C.c_float(float(s)), _p(y, C.c_float)),
           "fake_quantize")
    return y


def ema_update(ema_prev, initialized: bool, amax, decay) -> np.float32:
    """One step of the moving average of max|x| under Eq. 4."""
    out = C.c_float()
    _check(lib().q8o_ema_update(C.c_float(float(ema_prev)), C.c_int(1 if initialized else 0), C.c_float(float(amax)),
                                C.c_float(float(decay)), C.byref(out)), "ema_update")
    return np.float32(out.value)


def ste_backward(grad_xq) -> np.ndarray:
    """Eq. 5: the gradient passes the fake quantization unchanged."""
    g = _f32(grad_xq)
    out = np.empty(g.shape, dtype=np.float32)
    lib().q8o_ste_backward(_p(g, C.c_float), C.c_int64(g.size), _p(out, C.c_float))
    return out


def layernorm(a, gamma, beta, eps=1e-12, residual=None) -> np.ndarray:
    """LayerNorm over the last axis of a (+ residual), fp64 inside, one rounding to fp32 (Section 3: stays FP32)."""
    a = _f32(a)
    M, H = a.shape
    r = _f32(residual) if residual is not None else None
    y = np.empty((M, H), dtype=np.float32)
    _check(lib().q8o_layernorm(_p(a, C.c_float), _p(r, C.c_float) if r is not None else None, _p(_f32(gamma), C.c_float),
                               _p(_f32(beta), C.c_float), C.c_double(float(eps)), C.c_int64(M), C.c_int64(H),
                               _p(y, C.c_float)), "layernorm")
    return y

def attention(qkv, B: int, S: int, heads: int, d: int, mask=None, scale=None, threads: int = 1) -> np.ndarray:
    """softmax(scale * Q K^T + mask) V per head on the fused projection output qkv [B*S, 3*heads*d]; fp64 inside."""
    qkv = _f32(qkv)
    assert qkv.shape == (B * S, 3 * heads * d)
    mk = _f32(mask).reshape(B, S) if mask is not None else None
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    ctx = np.empty((B * S, heads * d), dtype=np.float32)
    _check(lib().q8o_attention(_p(qkv, C.c_float), C.c_int64(B), C.c_int64(S), C.c_int64(heads), C.c_int64(d),
                               _p(mk, C.c_float) if mk is not None else None, C.c_double(float(scale)),
                               _p(ctx, C.c_float), C.c_int(threads)), "attention")
    return ctx


def quantize_tensor(x):
    """Dynamic per-tensor quantization: S = 127 / max|x| (Eq. 3), then Eq. 1."""
    s = scale(absmax(x))
    return quantize(x, s), s


def linear(x, wq, sw, b=None, sx=None, act_gelu: bool = False, threads: int = 1) -> dict:
    """The quantized FC layer at inference, step by step (Section 3 + Section 4.1).

    x fp32 [M,K]; wq int8 [N,K] with scale(s) sw (one per column group); b fp32 [N] or None.
    sx None -> dynamic scale from this x; otherwise the stored (static) scale.
    Returns every intermediate: sx, xq, bq, acc (post-bias int32), y (fp32; after GELU if asked).
    """
    x = _f32(x)
    if sx is None:
        sx = scale(absmax(x))
    xq = quantize(x, sx)
    N = wq.shape[0]
    bq = quantize_bias(b, N, sx, sw)
    acc = gemm_i8(xq, wq, bq, threads=threads)
    y = dequant(acc, sx, sw)
    if act_gelu:
        y = gelu(y)
    return dict(sx=np.float32(sx), xq=xq, bq=bq, acc=acc, y=y)
