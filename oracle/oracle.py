"""fp64 CPU oracle for the column-split fully-connected + softmax cross-entropy head.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
It shares no code with the HIP library and never imports it.

What it computes.  The paper's motivating classifier (Section 1; Section 2.1,
"Tensor Model Parallelism" and the hybrid image-classification example; the
replicate/split listing of Section 3.1.2) is `logits = FC(features)` followed by
`Softmax(logits)`, with the FC weight cut along its class dimension
(ShardingInfo [0, 1] in the notation of Section 3.2.2) into shards whose widths
may be uneven (Section 3.3.1).  A split matmul is by definition the set of
matmuls on the column slices whose concatenation is the full product
(Section 2.1), so the sharded method reaches exactly the unsharded result up to
rounding order.  The oracle is therefore the plain, unsharded definition in
float64, plus the per-shard quantities written straight from their definitions.

The paper states neither the loss nor the backward pass; the reading taken is
softmax cross-entropy against integer labels, with gradient scale g
(g = 1 is the gradient of the summed loss, g = 1/B of the mean).

Notation: B rows, D features, C classes; X [B, D]; W [C, D] (class-major, i.e.
the paper's [D, C] matrix stored transposed); b [C]; y [B] integer labels;
shard s covers classes [o, o + C_s).

Pins (tests/test_oracle_pins.py): closed forms (uniform logits -> ln C, a
hand-worked 3-class example, the two-class logistic case), invariants (gradient
rows sum to zero, bias-shift invariance, linearity in g), partition invariance,
central finite differences, scipy's logsumexp, and a pure-Python loop version.
Every function below is pinned by at least one of them.
"""
import numpy as np

_F = np.float64


def _as64(a):
    return np.asarray(a, dtype=_F)


def logits(X, W, b=None):
    """Z[i, c] = sum_d X[i, d] * W[c, d] + b[c]   (Section 2.1: the matmul that is split)."""
    Z = _as64(X) @ _as64(W).T
    if b is not None:
        Z = Z + _as64(b)[None, :]
    return Z


def logsumexp_rows(Z):
    """lse_i = m_i + log(sum_c exp(Z_ic - m_i)) with m_i = max_c Z_ic."""
    m = Z.max(axis=1)
    return m + np.log(np.exp(Z - m[:, None]).sum(axis=1))


def unsharded(X, W, b, y, g=1.0, want_dW=True):
    """Softmax cross-entropy of the whole layer and all its gradients.

    Returns a dict with
      lse [B], loss [B], loss_mean (scalar),
      dZ [B, C] = g * (softmax(Z) - onehot(y)),
      dX [B, D] = dZ @ W,  dW [C, D] = dZ.T @ X,  db [C] = column sums of dZ.
    With want_dW=False the [C, D] product is left out (None): for a very wide layer it is the one
    output that does not fit a host comfortably.
    """
    X = _as64(X)
    W = _as64(W)
    y = np.asarray(y, dtype=np.int64)
    B = X.shape[0]
    Z = logits(X, W, b)
    lse = logsumexp_rows(Z)
    loss = lse - Z[np.arange(B), y]
    P = np.exp(Z - lse[:, None])
    dZ = P
    dZ[np.arange(B), y] -= 1.0
    dZ *= g
    return {
        "lse": lse,
        "loss": loss,
        "loss_mean": loss.mean() if B else _F(0.0),
        "dZ": dZ,
        "dX": dZ @ W,
        "dW": dZ.T @ X if want_dW else None,
        "db": dZ.sum(axis=0),
    }


def membership(y, class_offset, C_shard):
    """Integer part of the method: which rows' labels fall in the shard, and where.

    in_shard_i = (o <= y_i < o + C_s);  local_i = y_i - o (only meaningful when in_shard).
    """
    y = np.asarray(y, dtype=np.int64)
    in_shard = (y >= class_offset) & (y < class_offset + C_shard)
    local = y - class_offset
    return in_shard, local


def partials(X, W_s, b_s, y, class_offset):
    """Row statistics one shard contributes (the forward call of the split layer).

    m_i = max over the shard's classes of Z_ic,
    s_i = sum over the shard's classes of exp(Z_ic - m_i),
    t_i = Z_{i, y_i} if the label lies in the shard, else exactly 0.
    """
    Z = logits(X, W_s, b_s)
    B, C_s = Z.shape
    m = Z.max(axis=1)
    s = np.exp(Z - m[:, None]).sum(axis=1)
    in_shard, local = membership(y, class_offset, C_s)
    t = np.zeros(B, dtype=_F)
    rows = np.nonzero(in_shard)[0]
    t[rows] = Z[rows, local[rows]]
    return m, s, t


def combine(m_list, s_list, t_list):
    """Merge shard statistics into the unsharded log-sum-exp and loss.

    m = max_s m^s;  S = sum_s s^s * exp(m^s - m);  lse = m + log S;
    t = sum_s t^s;  loss = lse - t.
    """
    M = np.stack([_as64(a) for a in m_list])  # [S, B]
    S = np.stack([_as64(a) for a in s_list])
    T = np.stack([_as64(a) for a in t_list])
    m = M.max(axis=0)
    tot = (S * np.exp(M - m[None, :])).sum(axis=0)
    lse = m + np.log(tot)
    loss = lse - T.sum(axis=0)
    return lse, loss


def shard_grads(X, W_s, b_s, lse, y, class_offset, g=1.0):
    """Backward call of one shard, given the combined log-sum-exp.

    dZ_s[i, c] = g * (exp(Z_ic - lse_i) - [y_i == o + c]);
    dX_partial = dZ_s @ W_s;  dW_s = dZ_s.T @ X;  db_s = column sums of dZ_s.
    """
    X = _as64(X)
    W_s = _as64(W_s)
    Z = logits(X, W_s, b_s)
    B, C_s = Z.shape
    dZ = np.exp(Z - _as64(lse)[:, None])
    in_shard, local = membership(y, class_offset, C_s)
    rows = np.nonzero(in_shard)[0]
    dZ[rows, local[rows]] -= 1.0
    dZ *= g
    return {"dZ": dZ, "dX_partial": dZ @ W_s, "dW": dZ.T @ X, "db": dZ.sum(axis=0)}


def unsharded_chunked(X, W, b, y, g=1.0, rows_per_chunk=512, want_dW=True):
    """`unsharded` evaluated over row blocks, for shapes whose [B, C] float64 logits
    do not fit host memory.  Rows are independent in everything but dW and db,
    which are sums over rows and are accumulated block by block.  dZ is not kept.
    """
    X = _as64(X)
    W = _as64(W)
    y = np.asarray(y, dtype=np.int64)
    B, D = X.shape
    C = W.shape[0]
    lse = np.empty(B, dtype=_F)
    loss = np.empty(B, dtype=_F)
    dX = np.empty((B, D), dtype=_F)
    dW = np.zeros((C, D), dtype=_F) if want_dW else None
    db = np.zeros(C, dtype=_F)
    for r0 in range(0, B, rows_per_chunk):
        r1 = min(B, r0 + rows_per_chunk)
        part = unsharded(X[r0:r1], W, b, y[r0:r1], g, want_dW=want_dW)
        lse[r0:r1] = part["lse"]
        loss[r0:r1] = part["loss"]
        dX[r0:r1] = part["dX"]
        if want_dW:
            dW += part["dW"]
        db += part["db"]
    return {"lse": lse, "loss": loss, "loss_mean": loss.mean() if B else _F(0.0),
            "dX": dX, "dW": dW, "db": db}


def predictions(X, W_s, b_s, lse):
    """The shard's columns of Softmax(logits) (the last line of the paper's split listing,
    Section 3.1.2), given the log-sum-exp over ALL classes: P[i, c] = exp(Z_ic - lse_i)."""
    return np.exp(logits(X, W_s, b_s) - _as64(lse)[:, None])


def sp2_partial_logits(X, W, d0, d1):
    """The other sharding pattern of the matmul (Section 3.2.2, SP2): both inputs cut along the
    contraction; the slice [d0, d1) contributes Z_s[i, c] = sum_{d0 <= d < d1} X[i, d] * W[c, d]
    for ALL classes."""
    return _as64(X)[:, d0:d1] @ _as64(W)[:, d0:d1].T


def sp2_reduce(Z_parts, b, y):
    """What the AllReduce of SP2 yields, then the loss: Z = sum_s Z_s + b; (lse, loss) per row."""
    Z = np.zeros_like(_as64(Z_parts[0]))
    for Zs in Z_parts:
        Z = Z + _as64(Zs)
    if b is not None:
        Z = Z + _as64(b)[None, :]
    lse = logsumexp_rows(Z)
    y = np.asarray(y, dtype=np.int64)
    return lse, lse - Z[np.arange(Z.shape[0]), y]


def sgd_update(W, b, dW, db, lr):
    """The last phase of a mini-batch (Section 2.1): the gradients, scaled by the learning rate, update
    the parameters.  Plain SGD: W - lr * dW, b - lr * db."""
    Wn = _as64(W) - lr * _as64(dW)
    bn = None if b is None else _as64(b) - lr * _as64(db)
    return Wn, bn


def top1(X, W_s, b_s, class_offset):
    """The shard's arg-max prediction: (max_c Z_ic, class_offset + argmax_c Z_ic), first maximum on ties."""
    Z = logits(X, W_s, b_s)
    idx = Z.argmax(axis=1)
    return Z[np.arange(Z.shape[0]), idx], idx + class_offset


def combine_top1(vals, classes):
    """Merge of the shards' candidates: larger logit, lower class id among equals."""
    vals, classes = np.stack(vals), np.stack(classes)
    best_v = vals.max(axis=0)
    masked = np.where(vals == best_v[None, :], classes, np.iinfo(np.int64).max)
    return best_v, masked.min(axis=0)
