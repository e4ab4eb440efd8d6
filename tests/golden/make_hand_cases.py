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
Case N1 (nTrans chain y = Norm(x + a Norm(h - x)), Norm(v) = v / sqrt(mean v^2), eps = 0)
    x = [[1, 2, 2]], h = [[4, 6, 2]], a = [1, 1/2, 3]
    h - x = [3, 4, 0], mean square 25/3, Norm = [3, 4, 0] * sqrt(3)/5
    u = [1 + 3 sqrt(3)/5, 2 + 2 sqrt(3)/5, 2]; y = u / sqrt((u0^2 + u1^2 + u2^2) / 3)
Case G1 (gate of the GatedMLP block, SiLU(v) = v / (1 + exp(-v)), Y = SiLU(gate) * up), H = 4
    Z = [[0, ln 3, -ln 3, ln 7 | 5, 2, 4, -1]]
    exp(-ln 3) = 1/3 -> SiLU = (3/4) ln 3;  exp(ln 3) = 3 -> SiLU = -(1/4) ln 3;  exp(-ln 7) = 1/7 -> (7/8) ln 7
    Y = [0, (3/2) ln 3, -ln 3, -(7/8) ln 7]
Case G2 (the whole gated block on case H1's inputs, H = 1: gate = column 0, up = column 1 of H1)
    row 0: SiLU(3 sqrt(3)/5) * 8 sqrt(3)/5;  row 1: SiLU(sqrt(3)) * 2/sqrt(3)   (exp in 40-digit decimals)
Case Q1 (QKNorm in front of attention: layer normalisation of query and keys, eps = 0, then attention), D = 2
    q = [3, 1], gq = [1, 1], bq = [1/2, 0];  keys [2, 0] and [0, 5], gk = [1, 1], bk = [0, 0];  values [1, 0] and [0, 1]
    a vector of two components normalises to (+1, -1) or (-1, +1): qn = [1 + 1/2, -1], kn_1 = [1, -1], kn_2 = [-1, 1]
    scores +-(3/2 + 1) / sqrt(2); weights 1 / (1 + exp(-+5 / sqrt 2)); output = [w1, w2]
"""
from decimal import Decimal, getcontext
import os

getcontext().prec = 40
s3 = Decimal(3).sqrt()
h1 = [[3 * s3 / 5, 8 * s3 / 5], [s3, 2 / s3]]
r = (Decimal(17) / Decimal(3)).sqrt()
h3 = [[Decimal(4) / 3, Decimal(4) / 3], [Decimal(0), 1 / r]]

ln3, ln7 = Decimal(3).ln(), Decimal(7).ln()
g1 = [[Decimal(0), Decimal(3) / 2 * ln3, -ln3, -Decimal(7) / 8 * ln7]]
silu = lambda v: v / (1 + (-v).exp())
g2 = [[silu(h1[0][0]) * h1[0][1]], [silu(h1[1][0]) * h1[1][1]]]

nu = [1 + 3 * s3 / 5, 2 + 2 * s3 / 5, Decimal(2)]
nr = ((nu[0] ** 2 + nu[1] ** 2 + nu[2] ** 2) / 3).sqrt()
n1 = [[v / nr for v in nu]]

x = Decimal(5) / Decimal(2).sqrt()
q1 = [[1 / (1 + (-x).exp()), 1 / (1 + x.exp())]]

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hand_cases.txt")
with open(out, "w") as f:
    f.write("# Hand-computed cases for Eq. 1 (RMSNorm) followed by the MatMul of Fig. 2a (H1, H3)\n")
    f.write("# for the gate of the GatedMLP block (G1, G2), for the nTrans chain (N1) and for QKNorm in\n")
    f.write("# front of attention (Q1).\n")
    f.write("# Closed forms are derived in make_hand_cases.py; values to 30 digits.\n")
    f.write("# format: case row col value\n")
    for name, tab in (("H1", h1), ("H3", h3), ("G1", g1), ("G2", g2), ("N1", n1), ("Q1", q1)):
        for i, row in enumerate(tab):
            for j, v in enumerate(row):
                f.write(f"{name} {i} {j} {v:.30f}\n")
print(open(out).read())
