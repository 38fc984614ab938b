"""Reproduces the coefficients of gelu_erf() in zq_device.h.

GeLU(u) = max(u, 0) - a * Phi(-a) with a = |u|.  The kernel evaluates Phi(-a) as 2^P(a), P a
polynomial of degree 6 in a on [0, A]; this script fits P to log2 Phi(-a) so that the largest error of
a * Phi(-a) is smallest (iteratively reweighted least squares on Chebyshev nodes), with P(0) = -1 held
exact, then evaluates the fp32 Horner form on a dense grid and prints the errors.

    python gelu_exponent_fit.py          # needs numpy and scipy; not used at build or run time
"""
import numpy as np
from scipy.special import log_ndtr

DEG, A = 6, 5.6


def fit(deg=DEG, a_max=A, nodes=6000, iters=100):
    xs = np.cos(np.pi * (np.arange(nodes) + 0.5) / nodes) * a_max / 2 + a_max / 2
    target = log_ndtr(-xs) / np.log(2.0)
    w = xs * np.exp(log_ndtr(-xs)) + 1e-10          # d(a * Phi) = a * Phi * ln2 * dP
    wt = w.copy()
    full = np.vander(xs, deg + 1, increasing=True)
    for _ in range(iters):
        c, *_ = np.linalg.lstsq(full[:, 1:] * wt[:, None], (target + 1.0) * wt, rcond=None)
        c = np.concatenate([[-1.0], c])
        e = np.abs((full @ c - target) * w)
        wt = wt * (1 + 2.0 * e / e.max()) / 2
        wt *= w.mean() / wt.mean()
    return c


def gelu_fp32(c, u):
    c32 = c.astype(np.float32)
    a = np.minimum(np.abs(u), np.float32(A))
    p = np.full_like(a, c32[-1])
    for k in range(len(c) - 2, -1, -1):
        p = (p * a + c32[k]).astype(np.float32)
    h = np.exp2(p.astype(np.float64)).astype(np.float32)
    return np.maximum(u, 0).astype(np.float64) - a.astype(np.float64) * h.astype(np.float64)


if __name__ == "__main__":
    c = fit()
    for k, v in enumerate(c):
        print("c%d = %.8e  (0x%08x)" % (k, np.float32(v), int(np.float32(v).view(np.uint32))))
    u = np.concatenate([np.linspace(-12, 12, 4000001), [-65504.0, 65504.0]]).astype(np.float32)
    ref = u.astype(np.float64) * np.exp(log_ndtr(u.astype(np.float64)))
    err = np.abs(gelu_fp32(c, u) - ref)
    near = (np.abs(u) < 1) & (u != 0)
    print("max abs error %.3e at u = %g" % (err.max(), u[err.argmax()]))
    print("max rel error for |u| < 1: %.3e" % (err[near] / np.abs(ref[near])).max())
