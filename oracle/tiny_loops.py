"""Pure-Python loop version of the split softmax head, for problems of a few dozen
numbers.  TEST INFRASTRUCTURE ONLY.  It exists to cross-check oracle.py with code
that uses no array library: every sum is an explicit loop over the paper's indices
(Section 2.1 for the split matmul; Section 3.1.2 for FC followed by Softmax).
Python floats are IEEE double, so this is also float64.
"""
import math


def logits(X, W, b):
    B, C, D = len(X), len(W), len(X[0]) if X else 0
    Z = [[0.0] * C for _ in range(B)]
    for i in range(B):
        for c in range(C):
            acc = 0.0
            for d in range(D):
                acc += X[i][d] * W[c][d]
            Z[i][c] = acc + (b[c] if b is not None else 0.0)
    return Z


def forward_backward(X, W, b, y, g=1.0):
    """Returns (lse, loss, dX, dW, db) as nested lists."""
    B, C, D = len(X), len(W), len(X[0])
    Z = logits(X, W, b)
    lse, loss = [], []
    dZ = [[0.0] * C for _ in range(B)]
    for i in range(B):
        m = max(Z[i])
        tot = 0.0
        for c in range(C):
            tot += math.exp(Z[i][c] - m)
        lse_i = m + math.log(tot)
        lse.append(lse_i)
        loss.append(lse_i - Z[i][y[i]])
        for c in range(C):
            p = math.exp(Z[i][c] - lse_i)
            dZ[i][c] = g * (p - (1.0 if c == y[i] else 0.0))
    dX = [[0.0] * D for _ in range(B)]
    for i in range(B):
        for d in range(D):
            acc = 0.0
            for c in range(C):
                acc += dZ[i][c] * W[c][d]
            dX[i][d] = acc
    dW = [[0.0] * D for _ in range(C)]
    for c in range(C):
        for d in range(D):
            acc = 0.0
            for i in range(B):
                acc += dZ[i][c] * X[i][d]
            dW[c][d] = acc
    db = [0.0] * C
    for c in range(C):
        for i in range(B):
            db[c] += dZ[i][c]
    return lse, loss, dX, dW, db


def shard_partials(X, W, b, y, lo, hi):
    """(m, s, t) of the shard holding classes [lo, hi) of the full W, b."""
    Z = logits(X, W, b)
    m, s, t = [], [], []
    for i in range(len(X)):
        mi = -math.inf
        for c in range(lo, hi):
            if Z[i][c] > mi:
                mi = Z[i][c]
        si = 0.0
        for c in range(lo, hi):
            si += math.exp(Z[i][c] - mi)
        m.append(mi)
        s.append(si)
        t.append(Z[i][y[i]] if lo <= y[i] < hi else 0.0)
    return m, s, t
