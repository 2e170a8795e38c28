"""Regenerates and checks the constants of `gelu_erf` in csrc/q8_device.h (not imported by anything).

GELU(v) = max(v, 0) - |v| Q(|v|) with Q the upper tail of the standard normal distribution.
log2 Q(a) is fitted on [0, 6] by a degree-7 polynomial (least-squares fit in the Chebyshev basis on a
dense grid of the exact function); the script prints the power-basis coefficients as binary32 literals
and the worst GELU error of an fp32 evaluation against the binary64 definition.

    python -m paper_1910_06188_amd.gelu_fit
"""
import math

import numpy as np
from numpy.polynomial import chebyshev as cheb
from scipy.special import erfc, log_ndtr

A, DEG = 6.0, 7


def fit():
    a = np.linspace(0.0, A, 400001)
    c = cheb.chebfit(2 * a / A - 1, log_ndtr(-a) / math.log(2), DEG)
    power_u = cheb.cheb2poly(c)                      # in u = 2a/A - 1
    poly, u = np.poly1d([0.0]), np.poly1d([2 / A, -1])
    for k, ck in enumerate(power_u):
        poly = poly + ck * (u ** k)
    return poly.coeffs[::-1].astype(np.float32)      # ascending powers of a


def gelu32(v, co):
    v = v.astype(np.float32)
    a = np.minimum(np.abs(v), np.float32(A))
    p = np.full_like(a, co[-1])
    for ck in co[-2::-1]:
        p = (p * a + ck).astype(np.float32)
    return np.maximum(v, np.float32(0)) - (a * np.exp2(p).astype(np.float32)).astype(np.float32)


if __name__ == "__main__":
    co = fit()
    print("ascending coefficients:", ", ".join(f"{x:.9e}f" for x in co))
    v = np.linspace(-12, 12, 2400001)
    ref = 0.5 * v * erfc(-v / math.sqrt(2))
    err = np.abs(gelu32(v, co).astype(np.float64) - ref)
    print(f"max abs error {err.max():.3e}; worst error / (1e-6 + 1e-5 |ref|) = {(err / (1e-6 + 1e-5 * np.abs(ref))).max():.3f}")
