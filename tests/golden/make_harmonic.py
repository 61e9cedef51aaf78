"""Writes harmonic_scores.txt: closed-form accumulated post-vision attention for equal
logits (Sec. 3.2 with A'_ij = 1 / (m - tau + i + 1) on the causal region of Alg. 1)."""
from fractions import Fraction
import os

m, tau = 12, 4


def H(n):
    return sum(Fraction(1, x) for x in range(1, n + 1))


rows = [str(H(m) - H(max(j, m - tau))) for j in range(m)]
with open(os.path.join(os.path.dirname(__file__), "harmonic_scores.txt"), "w") as f:
    f.write(f"# m={m} tau={tau}; psi_j = H_m - H_max(j, m-tau), j = 0..m-1, exact fractions\n")
    f.write(" ".join(rows) + "\n")
