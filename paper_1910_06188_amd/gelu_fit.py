"""Regenerates and checks the constants of `gelu_erf` in csrc/q8_device.h (not imported by anything).

GELU(v) = max(v, 0) - |v| Q(|v|) with Q the upper tail of the standard normal distribution.
log2 Q(a) is fitted on [0, 6] by a degree-6 polynomial p.  An error dp in the exponent moves the GELU by
a Q(a) ln2 dp, so the fit minimises the largest value of  a Q(a) ln2 |p(a) - log2 Q(a)|  (Lawson's iteratively
re-weighted least squares in the Chebyshev basis on a dense grid): the exponent may be far off where a Q(a) is
tiny (a -> 0 and a -> 6) and is tight around a = 0.75 where a Q(a) peaks.  That buys more than one degree against
an unweighted fit.  The script prints the power-basis coefficients as binary32 literals and the worst GELU error
of an fp32 evaluation against the binary64 definition.

    python -m paper_1910_06188_amd.gelu_fit
"""
import math

import numpy as np
from numpy.polynomial import chebyshev as cheb
from scipy.special import erfc, log_ndtr, ndtr

A, DEG = 6.0, 6


def fit(iters=3000, n=12001):
    a = np.linspace(0.0, A, n)
    f = log_ndtr(-a) / math.log(2)
    w = a * ndtr(-a) * math.log(2) + 1e-12           # d GELU / d exponent
    V = cheb.chebvander(2 * a / A - 1, DEG)
    lam = np.full(n, 1.0 / n)
    best = (np.inf, None)
    for _ in range(iters):
        sw = np.sqrt(lam) * w
        c = np.linalg.lstsq(V * sw[:, None], f * sw, rcond=None)[0]
        e = np.abs(w * (V @ c - f))
        if e.max() < best[0]:
            best = (e.max(), c)
        lam = lam * e
        lam /= lam.sum()
    power_u = cheb.cheb2poly(best[1])                # in u = 2a/A - 1
    poly, u = np.poly1d([0.0]), np.poly1d([2 / A, -1])
    for k, ck in enumerate(power_u):
        poly = poly + ck * (u ** k)
    return poly.coeffs[::-1].astype(np.float32)      # ascending powers of a


def gelu32(v, co):
    v = v.astype(np.float32)
    a = np.minimum(np.abs(v), np.float32(A))
    p = np.full_like(a, co[-1])
    for ck in co[-2::-1]:                            # each step one fused multiply-add: a single rounding
        p = (p.astype(np.float64) * a + np.float64(ck)).astype(np.float32)
    e = np.exp2(p.astype(np.float64)).astype(np.float32)
    return (np.maximum(v, np.float32(0)).astype(np.float64) - a.astype(np.float64) * e).astype(np.float32)


if __name__ == "__main__":
    co = fit()
    print("ascending coefficients:", ", ".join(f"{x:.9e}f" for x in co))
    v = np.linspace(-12, 12, 2400001)
    ref = 0.5 * v * erfc(-v / math.sqrt(2))
    err = np.abs(gelu32(v, co).astype(np.float64) - ref)
    neg = err[v < 0].max()
    print(f"max abs error {err.max():.3e} (negative side {neg:.3e}); "
          f"worst error / (1e-6 + 1e-5 |ref|) = {(err / (1e-6 + 1e-5 * np.abs(ref))).max():.3f}")
