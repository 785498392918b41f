#!/usr/bin/env python3
"""Regenerates codebook_lloyd_max.txt: the 4-centroid Lloyd-Max quantisers (Eq. 3) of the level densities of
Lemma 2, f_l(psi) ~ sin^(2^(l-1)-1)(2 psi) on [0, pi/2], by fixed-point iteration with scipy quadrature.
Independent of the oracle and of the library (it imports neither).  Usage: python make_codebook_lloyd_max.py"""
import os

import numpy as np
from scipy.integrate import quad

HEADER = """# Lloyd-Max (continuous 1-D k-means, Eq. 3) codebooks with 4 centroids for the
# level densities of Lemma 2, f_l(psi) ~ sin^(2^(l-1)-1)(2 psi) on [0, pi/2].
# Written by make_codebook_lloyd_max.py (scipy quadrature, no oracle or library code);
# kept as a regression value.
# level  theta_0       theta_1       theta_2       theta_3       mean-squared-error
"""


def lloyd_max(m, K=4, tol=1e-13):
    f = lambda x: np.sin(2.0 * x) ** m
    total = quad(f, 0.0, np.pi / 2, epsabs=1e-14, epsrel=1e-14)[0]
    c = (np.arange(K) + 0.5) * (np.pi / 2) / K
    while True:
        edges = np.concatenate([[0.0], 0.5 * (c[:-1] + c[1:]), [np.pi / 2]])
        new = np.array([quad(lambda x: x * f(x), a, b, epsabs=1e-14, epsrel=1e-14)[0] /
                        quad(f, a, b, epsabs=1e-14, epsrel=1e-14)[0] for a, b in zip(edges[:-1], edges[1:])])
        if np.max(np.abs(new - c)) < tol:
            break
        c = new
    mse = sum(quad(lambda x, ck=ck: (x - ck) ** 2 * f(x), a, b, epsabs=1e-14, epsrel=1e-14)[0]
              for ck, a, b in zip(c, edges[:-1], edges[1:])) / total
    return c, mse


if __name__ == "__main__":
    lines = []
    for level in (2, 3, 4):
        c, mse = lloyd_max(2 ** (level - 1) - 1)
        lines.append(f"{level}  " + "  ".join(f"{v:.10f}" for v in c) + f"  {mse:.4e}".replace("e-03", "e-3"))
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "codebook_lloyd_max.txt")
    with open(out, "w") as fh:
        fh.write(HEADER + "\n".join(lines) + "\n")
    print(open(out).read())
