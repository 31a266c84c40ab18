"""Writes expected_byzantine_votes.txt: the closed form for E[q_hat] printed in the proof of
Theorem 1 (Appendix A.1), E[q_hat] = (p/r) * sum_{i=0}^{(r-1)/2} C(q, r-i) C(p-q, i) / C(p, r),
evaluated with exact integer binomials.  Uses nothing but the Python standard library."""
from fractions import Fraction
from math import comb
import os

CASES = [(45, 5, 3), (105, 10, 5), (15, 2, 3), (9, 1, 3), (30, 9, 3), (35, 10, 7)]

lines = ["# n(=p)  q  r  E[q_hat]   -- Appendix A.1, proof of Theorem 1 (general r);",
         "# for r = 3 it equals (p/3) q(q-1)(3p-2q-2) / (p(p-1)(p-2)), the lemma that follows it."]
for p, q, r in CASES:
    e = Fraction(p, r) * sum(comb(q, r - i) * comb(p - q, i) for i in range((r - 1) // 2 + 1)) / comb(p, r)
    if r == 3:
        assert e == Fraction(p, 3) * Fraction(q * (q - 1) * (3 * p - 2 * q - 2), p * (p - 1) * (p - 2))
    lines.append(f"{p} {q} {r} {float(e):.12f}")
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "expected_byzantine_votes.txt"), "w") as fh:
    fh.write("\n".join(lines) + "\n")
