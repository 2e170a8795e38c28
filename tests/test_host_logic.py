"""Checks, on the CPU, of arithmetic identities the HIP kernels rely on (the kernels themselves are
checked against the oracle on the GPU)."""
import numpy as np

from oracle import q8_oracle as O


def test_add_below_half_then_truncate_is_round_half_away():
    """The kernels round Eq. 1's bracket as trunc(p + copysign(0.5 - 2^-25, p)).  Against the oracle's
    trunc / compare-the-fraction definition: every float of [0.25, 4) and its negative, every tie and both
    neighbours of every tie up to 2^23, and a random sample of the rest."""
    c = np.nextafter(np.float32(0.5), np.float32(0))
    assert c == np.float32(0.49999997)

    def trick(p):
        return np.trunc((p + np.copysign(c, p)).astype(np.float32))

    def oracle_round(p):
        # Quantize with S = 1 clamps at +-127, so compare through it only inside the range
        return O.quantize(p, 1.0).astype(np.float32)

    lo, hi = np.float32(0.25).view(np.uint32), np.float32(4.0).view(np.uint32)       # 2^25 floats
    dense = np.arange(lo, hi, dtype=np.uint32).view(np.float32)
    for p in (dense, -dense):
        np.testing.assert_array_equal(trick(p), oracle_round(p))
    ties = np.arange(0, 126, dtype=np.float32) + np.float32(0.5)
    for p in (ties, np.nextafter(ties, np.float32(0)), np.nextafter(ties, np.float32(1000))):
        for sgn in (1, -1):
            q = (sgn * p).astype(np.float32)
            np.testing.assert_array_equal(trick(q), oracle_round(q))
    g = np.random.default_rng(11)
    r = (g.standard_normal(2_000_000) * 40).astype(np.float32)
    r = r[np.abs(r) < 126.4]
    np.testing.assert_array_equal(trick(r), oracle_round(r))
    # beyond the clamp: the definition itself (the oracle's clamp would hide the integer)
    big = np.concatenate([np.ldexp(ties[:64], 16), np.float32([2 ** 23 - 0.5, 2 ** 23 + 1, 2 ** 24 + 2, 3e9, 1e30])]).astype(np.float32)
    for q in (big, -big):
        t = np.trunc(q)
        ref = np.where(np.abs(q - t) >= np.float32(0.5), t + np.copysign(np.float32(1), q), t)
        np.testing.assert_array_equal(trick(q), ref)


def _gelu_constants_from_header():
    """The polynomial of gelu_erf as it stands in csrc/q8_device.h: highest power first."""
    import os
    import re
    here = os.path.dirname(os.path.abspath(__file__))
    src = open(os.path.join(here, "..", "paper_1910_06188_amd", "csrc", "q8_device.h")).read()
    body = src[src.index("float gelu_erf(float v)"):]
    body = body[:body.index("return")]
    first = re.search(r"__builtin_fmaf\((-?[0-9.e+-]+)f, a, (-?[0-9.e+-]+)f\)", body)
    rest = re.findall(r"__builtin_fmaf\(p, a, (-?[0-9.e+-]+)f\)", body)
    clamp = re.search(r"__builtin_fabsf\(v\), ([0-9.]+)f\)", body)
    return [np.float32(first.group(1)), np.float32(first.group(2))] + [np.float32(c) for c in rest], np.float32(clamp.group(1))


def test_gelu_polynomial_of_the_kernels_meets_the_tolerance_on_the_cpu():
    """GELU(v) = max(v, 0) - |v| 2^p(|v|) with the kernel's own constants, evaluated in emulated binary32 (each
    Horner step one fused multiply-add, i.e. a single rounding), against the oracle's binary64 erfc form on
    every multiple of 2^-16 in [-12, 12]: within abs 1e-6 + rel 1e-5, the bar of the GPU tests, with margin."""
    co, clamp = _gelu_constants_from_header()
    assert len(co) == 7 and clamp == np.float32(6.0)
    v = (np.arange(-12 * 65536, 12 * 65536 + 1, dtype=np.int64) / 65536.0).astype(np.float32)
    a = np.minimum(np.abs(v), clamp)
    p = np.full_like(a, co[0])
    for c in co[1:]:
        p = (p.astype(np.float64) * a.astype(np.float64) + np.float64(c)).astype(np.float32)
    e = np.exp2(p.astype(np.float64)).astype(np.float32)
    got = (np.maximum(v, np.float32(0)).astype(np.float64) - a.astype(np.float64) * e.astype(np.float64)).astype(np.float32)
    ref = O.gelu(v).astype(np.float64)
    ratio = np.abs(got.astype(np.float64) - ref) / (1e-6 + 1e-5 * np.abs(ref))
    assert ratio.max() < 0.2, ratio.max()
    assert np.abs(got.astype(np.float64) - ref)[v < 0].max() < 2e-7


def test_gelu_constants_are_what_the_fit_script_prints():
    """The constants in the header are reproducible: the weighted fit beside the package gives them again (to a few
    binary32 ulps: the fit is iterative, and a different BLAS threading may move its last bits)."""
    from paper_1910_06188_amd import gelu_fit
    co, clamp = _gelu_constants_from_header()
    fitted = gelu_fit.fit()                        # ascending powers
    assert clamp == np.float32(gelu_fit.A) and len(fitted) == gelu_fit.DEG + 1 == len(co)
    np.testing.assert_allclose(np.array(co[::-1], dtype=np.float64), fitted.astype(np.float64), rtol=2e-6, atol=0)
