"""Derives the polynomial behind erf_1b() in compress.hip:  erf(x) = sign(x) (1 - 2^(t P(t))),  t = min(|x|, 4),
with t P(t) fitted to log2(erfc(t)) on [0, 4] by iteratively re-weighted least squares on Chebyshev nodes (the weight
erfc(t) ln 2 turns an error of the exponent into the absolute error of erf, which is what is minimised).  Prints the
float32 coefficients and the largest absolute error of the float32 evaluation against scipy's erf on a dense grid.
Run by hand when the constants are to be re-derived; nothing imports it."""
import numpy as np
from scipy.special import erf, erfc

T, DEG = 4.0, 8


def fit(deg=DEG, iters=30, nodes=4000):
    t = 0.5 * T * (1 - np.cos(np.pi * (np.arange(nodes) + 0.5) / nodes))
    target, w = np.log2(erfc(t)), erfc(t) * np.log(2)
    wt = w.copy()
    A = np.stack([t ** (k + 1) for k in range(deg + 1)], axis=1)
    for _ in range(iters):
        c, *_ = np.linalg.lstsq(A * wt[:, None], target * wt, rcond=None)
        e = np.abs((A @ c - target) * w)
        wt = wt * np.sqrt(1 + 2.0 * e / e.max())
        wt /= wt.max()
    return c.astype(np.float32)


def evaluate_f32(c, x):
    t = np.minimum(np.abs(x), np.float32(T))
    p = np.full_like(t, c[-1])
    for k in range(len(c) - 2, -1, -1):
        p = (p * t + c[k]).astype(np.float32)
    e = (np.float32(1) - np.exp2((p * t).astype(np.float32)).astype(np.float32)).astype(np.float32)
    return np.copysign(e, x)


if __name__ == "__main__":
    c = fit()
    x = np.linspace(-6, 6, 2000001).astype(np.float32)
    err = np.abs(evaluate_f32(c, x).astype(np.float64) - erf(x.astype(np.float64)))
    print("coefficients c0..c%d:" % DEG, ", ".join("%.9ef" % v for v in c))
    print("max abs error of the float32 evaluation: %.3e at x = %g" % (err.max(), x[err.argmax()]))
