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
