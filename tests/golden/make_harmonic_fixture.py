"""Writes harmonic_uniform_attention.txt: exact values of the forgotten score under uniform
causal attention (Q = 0 => P[i, j] = 1/(i+1) for j <= i), from Section 3.3 Eq.5 with exact
rational arithmetic.  At alpha = 1 this is H_n - H_j (harmonic numbers)."""
from fractions import Fraction
import os

n = 12
lines = ["# n alpha_num alpha_den j  S_j_num S_j_den"]
for a in (Fraction(1), Fraction(1, 2)):
    for j in range(n):
        s = sum(a ** (n - 1 - i) * Fraction(1, i + 1) for i in range(j, n))
        lines.append(f"{n} {a.numerator} {a.denominator} {j} {s.numerator} {s.denominator}")
with open(os.path.join(os.path.dirname(__file__), "harmonic_uniform_attention.txt"), "w") as f:
    f.write("\n".join(lines) + "\n")
