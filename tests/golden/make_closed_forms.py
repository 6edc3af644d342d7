"""Regenerates uniform_scores_closed_form.txt from exact arithmetic (mpmath, 50 digits).
Calls nothing but mpmath: the values are a closed form, independent of every implementation."""
import os

from mpmath import binomial, log, mp

mp.dps = 50
HEADER = """\
# Closed form, not a paper value: with all output scores equal (W_out = 0, b_out = 0) every
# emission has probability 1/V, every alignment of a (T, U) lattice emits exactly T blanks and
# U labels, and there are C(T+U-1, U) alignments (the last emission is always the blank at
# (T-1, U)), hence   -ln P(y|x) = (T + U) ln V - ln C(T+U-1, U)   (Section 2: L = -sum_b ln P).
# Columns: T U V loss       (exact integer binomials, 50-digit logarithms, printed to 17 digits)
"""
CASES = [(20, 5, 16), (1, 0, 3), (7, 3, 5), (250, 50, 1024), (1000, 200, 1024), (800, 240, 8192)]

if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "uniform_scores_closed_form.txt")
    with open(path, "w") as f:
        f.write(HEADER)
        for T, U, V in CASES:
            val = (T + U) * log(V) - log(binomial(T + U - 1, U))
            f.write(f"{T} {U} {V} {mp.nstr(val, 17)}\n")
