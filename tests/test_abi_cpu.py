"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "q8.h")
LIB = os.path.join(ROOT, "paper_1910_06188_amd", "libq8.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_1910_06188_amd import build
        build.build()
    return C.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(q8_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for n in ("q8_absmax", "q8_quantize", "q8_linear", "q8_embedding"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_version_and_status_strings(lib):
    lib.q8_version.restype = C.c_char_p
    lib.q8_status_str.restype = C.c_char_p
    assert b"gfx950" in lib.q8_version()
    texts = {lib.q8_status_str(i) for i in range(7)}
    assert len(texts) == 7


def test_host_side_argument_checks(lib):
    vp, i64 = C.c_void_p, C.c_int64
    lib.q8_absmax.argtypes = [vp, i64, vp, vp, vp]
    lib.q8_quantize.argtypes = [vp, i64, vp, vp, vp]
    lib.q8_linear.argtypes = [vp, vp, vp, vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, vp, C.c_uint32, vp]
    lib.q8_embedding.argtypes = [vp, vp, i64, i64, vp, i64, vp, C.c_int, vp, vp]
    OK, NULL, SHAPE, ALIGN, FLAGS = 0, 1, 2, 3, 4
    p = 0x1000  # never dereferenced on the host
    assert lib.q8_absmax(p, -1, p, p + 4, None) == SHAPE
    assert lib.q8_absmax(None, 8, p, p + 4, None) == NULL
    assert lib.q8_absmax(p, 8, None, p + 4, None) == NULL
    assert lib.q8_absmax(p + 2, 8, p, p + 4, None) == ALIGN
    assert lib.q8_quantize(p, -5, p, p, None) == SHAPE
    assert lib.q8_quantize(p, 0, None, None, None) == OK          # empty: nothing to do
    assert lib.q8_quantize(p, 4, None, p, None) == NULL
    # linear: K above the int32-safe bound, groups not dividing N, unknown flag, flag without its pointer
    assert lib.q8_linear(p, p, None, p, p, 1, 4, 4, 131072, p, None, None, None, 0, None) == SHAPE
    assert lib.q8_linear(p, p, None, p, p, 3, 4, 4, 128, p, None, None, None, 0, None) == SHAPE
    assert lib.q8_linear(p, p, None, p, p, 1, 4, 4, 128, p, None, None, None, 8, None) == FLAGS
    assert lib.q8_linear(p, p, None, p, p, 1, 4, 4, 128, p, None, None, None, 2, None) == FLAGS
    assert lib.q8_linear(p, p, None, p, p, 1, 4, 4, 128, p, None, None, None, 4, None) == FLAGS
    assert lib.q8_linear(p, None, None, p, p, 1, 4, 4, 128, p, None, None, None, 0, None) == NULL
    assert lib.q8_linear(p, p, None, p, p, 1, 0, 4, 128, p, None, None, None, 0, None) == OK   # M = 0
    assert lib.q8_linear(p, p, None, p + 2, p, 1, 4, 4, 128, p, None, None, None, 0, None) == ALIGN
    assert lib.q8_embedding(p, p, 10, 8, None, 4, p, 0, None, None) == NULL
    assert lib.q8_embedding(p, p, 10, 8, p, 0, p, 0, None, None) == OK                       # T = 0
    assert lib.q8_embedding(p, p, -1, 8, p, 4, p, 0, None, None) == SHAPE
    # three-table lookup: a table with rows needs its pointer; an empty one may be null (its ids are all bad)
    lib.q8_embedding_sum3.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp, vp, vp]
    assert lib.q8_embedding_sum3(p, 4, p, 4, None, 2, p, 8, p, p, p, 3, p, None, None) == NULL
    assert lib.q8_embedding_sum3(p, 4, p, 4, None, 0, p, 8, p, p, p, 0, p, None, None) == OK          # T = 0
    assert lib.q8_embedding_sum3(p, 4, p, 4, p, -1, p, 8, p, p, p, 3, p, None, None) == SHAPE
    # training side: every check below returns before anything would be launched
    lib.q8_fake_quantize.argtypes = [vp, i64, vp, vp, vp]
    lib.q8_ema_update.argtypes = [vp, C.c_int, C.c_float, vp, vp, vp, vp]
    lib.q8_fake_quantize_ema.argtypes = [vp, i64, C.c_float, vp, vp, vp, vp]
    lib.q8_ste_backward.argtypes = [vp, i64, vp, vp]
    assert lib.q8_fake_quantize(p, -1, p, p, None) == SHAPE
    assert lib.q8_fake_quantize(p, 0, None, None, None) == OK
    assert lib.q8_fake_quantize(p, 4, None, p, None) == NULL
    assert lib.q8_fake_quantize(p, 4, p, p + 1, None) == ALIGN
    assert lib.q8_ema_update(p, 0, 0.5, p, None, None, None) == SHAPE
    assert lib.q8_ema_update(p, 1, 1.5, p, None, None, None) == SHAPE
    assert lib.q8_ema_update(p, 1, float("nan"), p, None, None, None) == SHAPE
    assert lib.q8_ema_update(p, 1, 0.5, None, None, None, None) == NULL
    assert lib.q8_fake_quantize_ema(p, 8, 0.5, p, None, p, None) == NULL
    assert lib.q8_fake_quantize_ema(p, 8, -0.1, p, p, p, None) == SHAPE
    assert lib.q8_ste_backward(p, 8, None, None) == NULL
    assert lib.q8_ste_backward(p, -2, p, None) == SHAPE
    assert lib.q8_ste_backward(p, 0, None, None) == OK
    # fused LayerNorm entry points
    lib.q8_layernorm_absmax.argtypes = [vp, vp, vp, vp, C.c_float, i64, i64, vp, vp, vp, vp, vp]
    lib.q8_embedding_sum3_layernorm.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp, vp, C.c_float, vp, vp, vp, vp, vp, vp]
    assert lib.q8_layernorm_absmax(p, None, p, p, 1e-12, -1, 4, p, None, None, None, None) == SHAPE
    assert lib.q8_layernorm_absmax(p, None, p, p, 1e-12, 4, 0, p, None, None, None, None) == SHAPE
    assert lib.q8_layernorm_absmax(p, None, p, p, -1.0, 4, 4, p, None, None, None, None) == SHAPE
    assert lib.q8_layernorm_absmax(None, None, p, p, 1e-12, 4, 4, p, None, None, None, None) == NULL
    assert lib.q8_layernorm_absmax(p, None, p, p, 1e-12, 4, 4, p, None, p, None, None) == NULL      # scale without codes
    assert lib.q8_layernorm_absmax(p, None, None, p, 1e-12, 4, 4, p, None, None, None, None) == NULL
    assert lib.q8_layernorm_absmax(p + 2, None, p, p, 1e-12, 1, 4, p, None, None, None, None) == ALIGN
    assert lib.q8_embedding_sum3_layernorm(p, 4, p, 4, p, 4, p, 4, None, p, p, 2, p, p, 1e-12, p, None, None, None, None, None) == NULL
    assert lib.q8_embedding_sum3_layernorm(p, 4, p, 4, p, 4, p, 0, p, p, p, 2, p, p, 1e-12, p, None, None, None, None, None) == SHAPE
    # the FC fed by abs-max slots
    lib.q8_linear_f32_slots.argtypes = [vp, vp, C.c_int, vp, vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, vp, vp, vp, C.c_uint32, vp]
    assert lib.q8_linear_f32_slots(p, None, 1, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == NULL
    assert lib.q8_linear_f32_slots(p, p, 0, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == SHAPE
    assert lib.q8_linear_f32_slots(p, p, 1, p, None, p, 1, 4, 4, 128, p, None, p, None, None, None, 0, None) == NULL
    assert lib.q8_linear_f32_slots(p, p + 2, 1, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == ALIGN
    assert lib.q8_linear_f32_slots(None, p, 1, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == NULL
    # the no-allocation variant refuses what its static scratch cannot hold before it touches the device
    lib.q8_linear_f32_static.argtypes = [vp, vp, vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, vp, C.c_uint32, vp]
    TOO_LARGE = 6
    assert lib.q8_linear_f32_static(p, p, None, p, 1, (64 << 20) // 1024 + 1, 8, 1024, p, None, None, None, 0, None) == TOO_LARGE
    assert lib.q8_linear_f32_static(p, p, None, p, 1, -1, 8, 1024, p, None, None, None, 0, None) == SHAPE
    assert lib.q8_linear_f32_static(p, p, None, p, 1, 4, 8, 128, p, p + 2, None, None, 0, None) == ALIGN
    # the FC layer with the residual addition fused: fp32 output only, the residual is required
    lib.q8_linear_residual.argtypes = [vp, vp, vp, vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, vp, C.c_uint32, vp]
    assert lib.q8_linear_residual(p, p, None, p, p, 1, 4, 4, 128, p, p, None, None, 4, None) == FLAGS
    assert lib.q8_linear_residual(p, p, None, p, p, 1, 4, 4, 128, None, p, None, None, 0, None) == NULL
    assert lib.q8_linear_residual(p, p, None, p, p, 1, 4, 4, 128, p + 2, p, None, None, 0, None) == ALIGN
    assert lib.q8_linear_residual(p, p, None, p, p, 1, 4, 4, 128, p, p, None, None, 2, None) == FLAGS   # abs-max without its slot
    assert lib.q8_linear_residual(None, None, None, None, None, 1, 0, 4, 128, None, None, None, None, 0, None) == 0
    # the dynamic quantizer on its own, and the measurement kernels' argument checks
    lib.q8_quantize_dynamic.argtypes = [vp, i64, vp, vp, vp, vp]
    assert lib.q8_quantize_dynamic(p, -1, p, p, None, None) == SHAPE
    assert lib.q8_quantize_dynamic(p, 8, p, None, None, None) == NULL
    assert lib.q8_quantize_dynamic(None, 8, p, p, None, None) == NULL
    assert lib.q8_quantize_dynamic(p + 2, 8, p, p, None, None) == ALIGN
    lib.q8_debug_mfma_rate.argtypes = [vp, C.c_int, C.c_int, vp, vp]
    lib.q8_debug_stream_copy.argtypes = [vp, vp, i64, vp]
    lib.q8_debug_loop_probe.argtypes = [C.c_int, vp, vp, C.c_int, vp, vp]
    assert lib.q8_debug_mfma_rate(None, 1, 1, p, None) == NULL
    assert lib.q8_debug_mfma_rate(p, -1, 1, p, None) == SHAPE
    assert lib.q8_debug_mfma_rate(p + 4, 1, 1, p, None) == ALIGN
    assert lib.q8_debug_stream_copy(p, p, 24, None) == SHAPE            # whole 16-byte units only
    assert lib.q8_debug_stream_copy(p, None, 32, None) == NULL
    assert lib.q8_debug_stream_copy(p, p, 0, None) == OK
    assert lib.q8_debug_loop_probe(3, p, p, 4, p, None) == FLAGS           # not one of the built combinations
    assert lib.q8_debug_loop_probe(7, None, p, 4, p, None) == NULL
    assert lib.q8_debug_loop_probe(7, p, p, -4, p, None) == SHAPE
    # FP32 attention between the QKV and attention-output FC layers
    lib.q8_attention.argtypes = [vp, i64, i64, C.c_int, C.c_int, vp, C.c_float, vp, vp, vp, vp, vp]
    assert lib.q8_attention(p, -1, 8, 2, 64, None, 0.125, p, None, None, None, None) == SHAPE
    assert lib.q8_attention(p, 1, 0, 2, 64, None, 0.125, p, None, None, None, None) == SHAPE
    assert lib.q8_attention(p, 1, 8, 0, 64, None, 0.125, p, None, None, None, None) == SHAPE
    assert lib.q8_attention(p, 1, 8, 2, 0, None, 0.125, p, None, None, None, None) == SHAPE
    assert lib.q8_attention(p, 1, 8, 2, 64, None, 0.0, p, None, None, None, None) == SHAPE
    assert lib.q8_attention(p, 1, 8, 2, 64, None, float("nan"), p, None, None, None, None) == SHAPE
    assert lib.q8_attention(None, 1, 8, 2, 64, None, 0.125, p, None, None, None, None) == NULL
    assert lib.q8_attention(p, 1, 8, 2, 64, None, 0.125, None, None, None, None, None) == NULL      # neither ctx nor codes
    assert lib.q8_attention(p, 1, 8, 2, 64, None, 0.125, p, None, p, None, None) == NULL            # scale without codes
    assert lib.q8_attention(p + 2, 1, 8, 2, 64, None, 0.125, p, None, None, None, None) == ALIGN
    assert lib.q8_attention(p, 1, 20000, 2, 48, None, 0.125, p, None, None, None, None) == SHAPE     # generic kernel: S <= 16384
    assert lib.q8_attention(None, 0, 8, 2, 64, None, 0.125, None, None, None, None, None) in (OK, 5)  # B = 0: nothing to read (no GPU here: launch may be refused)


def test_product_package_does_not_reach_the_oracle():
    """The product path must not import, link or read anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_1910_06188_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not re.search(r"(from|import)\s+oracle|q8_oracle|oracle/|q8o_", text), os.path.join(dirpath, f)
