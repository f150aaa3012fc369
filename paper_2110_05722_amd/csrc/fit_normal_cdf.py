"""Derives the polynomial used by normal_cdf() in bias_act_dropout.hip.

    python paper_2110_05722_amd/csrc/fit_normal_cdf.py

q(u) ~ log2(erfc(u / sqrt 2)) = log2(2 Phi(-u)) on [0, 6.5]: least squares on Chebyshev
nodes, degree 10, converted to the power basis in u (Horner order is printed highest
degree first).  Also prints the error of the fit in exact arithmetic and of its fp32
Horner evaluation, both relative to erfc.
"""
import numpy as np
from numpy.polynomial import chebyshev, polynomial
from scipy.special import erfc, log_ndtr

U, DEG = 6.5, 10


def log2_erfc(u):
    return (log_ndtr(-u) + np.log(2.0)) / np.log(2.0)


def main():
    nodes = np.cos(np.pi * (np.arange(20000) + 0.5) / 20000) * U / 2 + U / 2
    fit = chebyshev.Chebyshev.fit(nodes, log2_erfc(nodes), DEG, domain=[0, U])
    coef = fit.convert(kind=polynomial.Polynomial).coef.astype(np.float32)
    grid = np.linspace(0, U, 400001)
    print("fit, exact arithmetic: max relative error of erfc",
          float(np.abs(fit(grid) - log2_erfc(grid)).max() * np.log(2.0)))
    g32 = grid.astype(np.float32)
    acc = np.full_like(g32, coef[-1])
    for k in range(DEG - 1, -1, -1):
        acc = (acc * g32 + coef[k]).astype(np.float32)
    rel = np.abs(np.exp2(acc.astype(np.float64)) - erfc(g32.astype(np.float64) / np.sqrt(2.0)))
    rel /= erfc(g32.astype(np.float64) / np.sqrt(2.0))
    print("fp32 Horner: max relative error of erfc", float(rel.max()))
    for k in range(DEG, -1, -1):
        print(f"  u^{k:<2d} {coef[k]:.9e}f")


if __name__ == "__main__":
    main()
