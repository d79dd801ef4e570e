"""Writes tests/golden/uniform_attention_scores.txt with exact rational arithmetic.

With all-zero queries every visible key of row i gets probability 1/(M+i+1)
(chunk attention over [cache || chunk], Sec. 3.1 / Fig. 1 step 1, mask: row i
sees keys j <= M+i), so the attention-mass score of key j is
    G * sum_{i = max(j-M, 0, Ct-W)}^{Ct-1} 1/(M+i+1).
This script evaluates that sum with `fractions.Fraction` and prints 17
significant digits.  It imports nothing from this repository.
"""
from fractions import Fraction
import os

CASES = [  # (M, Ct, W, G)
    (0, 1, 0, 1), (0, 6, 0, 1), (5, 4, 0, 2), (7, 9, 3, 4), (3, 8, 1, 1), (12, 5, 5, 3),
]


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "uniform_attention_scores.txt"), "w") as f:
        f.write("# uniform-attention eviction scores, exact harmonic sums (see make_uniform_golden.py)\n")
        f.write("# line: M Ct W G : score[0..M+Ct)   (W = 0 means the whole chunk observes)\n")
        for M, Ct, W, G in CASES:
            w = Ct if W == 0 else W
            vals = []
            for j in range(M + Ct):
                lo = max(j - M, 0, Ct - w)
                s = sum((Fraction(1, M + i + 1) for i in range(lo, Ct)), Fraction(0))
                vals.append(G * s)
            f.write(f"{M} {Ct} {W} {G} : " + " ".join(f"{float(x):.17g}" for x in vals) + "\n")


if __name__ == "__main__":
    main()
