"""Writes tests/golden/hand_cases.txt from closed forms only (no oracle, no GPU).

Each case is small enough to do on paper; the expected values are the closed
forms below evaluated with 40-digit decimal arithmetic, so they depend on no
floating-point implementation of the method.

Case H1 (Eq. 1 of the case-study section followed by the product of Fig. 2a, eps = 0)
    X = [[3,4,0],[1,2,2]], G = [1,2,1/2], W = [[1,0],[0,1],[2,-2]]
    row 0: mean square 25/3, X*G = [3,8,0], times W = [3,8]  -> [3,8] / sqrt(25/3) = [3*sqrt(3)/5, 8*sqrt(3)/5]
    row 1: mean square 3,    X*G = [1,4,1], times W = [3,2]  -> [3,2] / sqrt(3)    = [sqrt(3), 2/sqrt(3)]
Case H3 (placement of eps: added to the mean square, under the root), eps = 5
    X = [[2,2,2],[-1,0,1]], G = [1,1,1], W = [[1,0],[0,1],[1,1]]
    row 0: sqrt(4 + 5) = 3            -> [4,4]/3
    row 1: sqrt(2/3 + 5) = sqrt(17/3) -> [0,1]/sqrt(17/3)
    (adding eps to the root instead would give 4/7 for row 0)
"""
from decimal import Decimal, getcontext
import os

getcontext().prec = 40
s3 = Decimal(3).sqrt()
h1 = [[3 * s3 / 5, 8 * s3 / 5], [s3, 2 / s3]]
r = (Decimal(17) / Decimal(3)).sqrt()
h3 = [[Decimal(4) / 3, Decimal(4) / 3], [Decimal(0), 1 / r]]

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hand_cases.txt")
with open(out, "w") as f:
    f.write("# Hand-computed cases for Eq. 1 (RMSNorm) followed by the MatMul of Fig. 2a.\n")
    f.write("# Closed forms are derived in make_hand_cases.py; values to 30 digits.\n")
    f.write("# format: case row col value\n")
    for name, tab in (("H1", h1), ("H3", h3)):
        for i, row in enumerate(tab):
            for j, v in enumerate(row):
                f.write(f"{name} {i} {j} {v:.30f}\n")
print(open(out).read())
