"""Derives the polynomial used by the gating kernel's normal CDF.

    erfc(x) = t * exp(-x^2 + P(t)),   t = 1 / (1 + x/2),   x >= 0

P is a degree-DEG polynomial in t fitted (Chebyshev nodes, least squares) to
f(t) = log(erfc(x) / t) + x^2 with x = 2 (1/t - 1); f is smooth on (0, 1] and an absolute error
in f is a relative error in erfc.  Run this script to regenerate the coefficients pasted into
gate.hip; it prints them together with the worst relative error of an fp32 evaluation.
"""
import numpy as np
from scipy.special import erfc, erfcx

DEG = 10


def f_of_t(t):
    x = 2.0 * (1.0 / t - 1.0)
    # log(erfc(x)) + x^2 = log(erfcx(x)) without underflow
    return np.log(erfcx(x)) - np.log(t)


def main():
    k = np.arange(4000)
    t = 0.5 * (1.0 + np.cos(np.pi * (k + 0.5) / k.size))      # Chebyshev nodes on (0, 1)
    t = np.clip(t, 1e-6, 1.0)
    cheb = np.polynomial.chebyshev.Chebyshev.fit(t, f_of_t(t), DEG, domain=[0.0, 1.0])
    poly = cheb.convert(kind=np.polynomial.Polynomial, domain=[0.0, 1.0], window=[0.0, 1.0])
    coef = poly.coef.astype(np.float32)
    # fp32 evaluation
    x = np.concatenate([np.linspace(0, 6, 600001), np.linspace(6, 13, 7001)]).astype(np.float32)
    tt = (np.float32(1.0) / (np.float32(1.0) + np.float32(0.5) * x)).astype(np.float32)
    p = np.zeros_like(tt) + coef[-1]
    for c in coef[-2::-1]:
        p = (p * tt + c).astype(np.float32)
    approx = (tt * np.exp((-(x * x) + p).astype(np.float32))).astype(np.float32)
    truth = erfc(x.astype(np.float64))
    ok = truth > 1e-37
    rel = np.abs(approx[ok].astype(np.float64) - truth[ok]) / truth[ok]
    print("degree", DEG, "max relative error (fp32 eval, erfc > 1e-37): %.3e" % rel.max())
    print("coefficients c0..c%d:" % DEG)
    print(", ".join("%.9ef" % c for c in coef))


if __name__ == "__main__":
    main()
