"""Writes tiny_rational.json: a 3x4, d=2 iALS half-epoch solved in exact rational arithmetic.

Independent of the oracle and of the GPU library: it forms the normal equations of
the paper's Eq. 4 with ``fractions.Fraction`` and solves them by Gaussian
elimination, then evaluates Eq. 3 as the literal double sum.  Run by hand:
``python tests/golden/make_tiny_rational.py``.
"""
import json
import os
from fractions import Fraction as F

H = [[F(1), F(2)], [F(-1), F(1, 2)], [F(0), F(3)], [F(2), F(-1)]]
rows = {0: [(0, F(1)), (2, F(1, 2))], 1: [], 2: [(1, F(2)), (2, F(1)), (3, F(3, 2))]}
alpha, lam = F(1, 4), F(1, 8)
d = 2


def solve2(A, b):
    det = A[0][0] * A[1][1] - A[0][1] * A[1][0]
    return [(b[0] * A[1][1] - A[0][1] * b[1]) / det, (A[0][0] * b[1] - A[1][0] * b[0]) / det]


W = []
for u in range(3):
    A = [[lam if a == c else F(0) for c in range(d)] for a in range(d)]
    b = [F(0)] * d
    for h in H:
        for a in range(d):
            for c in range(d):
                A[a][c] += alpha * h[a] * h[c]
    for i, y in rows[u]:
        for a in range(d):
            b[a] += y * H[i][a]
            for c in range(d):
                A[a][c] += H[i][a] * H[i][c]
    W.append(solve2(A, b))

loss = F(0)
for u in range(3):
    obs = dict(rows[u])
    for i in range(4):
        yhat = sum(W[u][a] * H[i][a] for a in range(d))
        loss += alpha * yhat * yhat
        if i in obs:
            loss += (obs[i] - yhat) ** 2
loss += lam * (sum(x * x for w in W for x in w) + sum(x * x for h in H for x in h))

indptr, indices, values = [0], [], []
for u in range(3):
    for i, y in rows[u]:
        indices.append(i)
        values.append(float(y))
    indptr.append(len(indices))
out = {
    "source": "exact rational solve of Eq. 4 / evaluation of Eq. 3 (make_tiny_rational.py)",
    "alpha": float(alpha), "lambda": float(lam), "indptr": indptr, "indices": indices, "values": values,
    "H": [[float(x) for x in h] for h in H],
    "W_solved": [[float(x) for x in w] for w in W],
    "W_solved_exact": [[str(x) for x in w] for w in W],
    "loss_at_solution": float(loss), "loss_exact": str(loss),
}
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_rational.json"), "w") as f:
    json.dump(out, f, indent=1)
