"""Pins for the fp64 oracle: closed forms, invariants, special cases, brute force.

None of these re-types the oracle's formula: each checks it against something the
mathematics fixes independently, chosen so that a dropped term, a wrong sign or
index, or a transposed operand fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import oracle, tiny_loops

RNG = lambda seed: np.random.Generator(np.random.PCG64(seed))


def _rand_problem(seed, B, D, C, scale=1.0, bias=True):
    r = RNG(seed)
    X = r.standard_normal((B, D)) * scale
    W = r.standard_normal((C, D)) * scale
    b = r.standard_normal(C) if bias else None
    y = r.integers(0, C, size=B)
    return X, W, b, y


# P1 -- uniform logits: lse = b + ln C, loss = ln C, dZ = 1/C - onehot.
@pytest.mark.parametrize("C", [2, 1000, 100_000])
def test_uniform_logits_closed_form(C):
    B, D = 5, 3
    X = RNG(1).standard_normal((B, D))
    W = np.zeros((C, D))
    b = np.full(C, 0.75)
    y = np.array([0, C - 1, C // 2, 1 % C, 0])
    out = oracle.unsharded(X, W, b, y)
    assert np.allclose(out["lse"], 0.75 + math.log(C), rtol=0, atol=1e-12)
    assert np.allclose(out["loss"], math.log(C), rtol=0, atol=1e-12)
    expect = np.full((B, C), 1.0 / C)
    expect[np.arange(B), y] -= 1.0
    assert np.allclose(out["dZ"], expect, rtol=0, atol=1e-15)
    assert np.allclose(out["dX"], 0.0, atol=1e-15)      # W = 0
    # dW[c, :] = sum_i dZ[i, c] X[i, :]
    cnt = np.zeros((C, D))
    np.add.at(cnt, y, X)
    assert np.allclose(out["dW"], X.sum(0)[None, :] / C - cnt, atol=1e-12)


def test_ln_values_printed():
    # the two constants the uniform case must hit for the workloads' class counts
    out = oracle.unsharded(np.ones((1, 1)), np.zeros((1000, 1)), None, np.array([3]))
    assert abs(out["loss"][0] - 6.907755278982137) < 1e-12
    out = oracle.unsharded(np.ones((1, 1)), np.zeros((100_000, 1)), None, np.array([3]))
    assert abs(out["loss"][0] - 11.512925464970229) < 1e-12


# P2 -- hand-worked example: x = 1, w = (0, ln 2, ln 3), y = 2.
def test_hand_example_three_classes():
    X = np.array([[1.0]])
    W = np.array([[0.0], [math.log(2.0)], [math.log(3.0)]])
    out = oracle.unsharded(X, W, None, np.array([2]))
    assert abs(out["lse"][0] - math.log(6.0)) < 1e-14
    assert abs(out["loss"][0] - math.log(2.0)) < 1e-14
    assert np.allclose(out["dZ"][0], [1 / 6, 1 / 3, -1 / 2], atol=1e-15)
    assert abs(out["dX"][0, 0] - (math.log(2.0) / 3 - math.log(3.0) / 2)) < 1e-14
    assert np.allclose(out["dW"][:, 0], [1 / 6, 1 / 3, -1 / 2], atol=1e-15)   # x = 1
    assert np.allclose(out["db"], [1 / 6, 1 / 3, -1 / 2], atol=1e-15)
    # an asymmetric version (x = 2, D = 2) that separates dW's two axes
    X = np.array([[2.0, -1.0]])
    W = np.array([[0.0, 0.0], [math.log(2.0) / 2, 0.0], [0.0, -math.log(3.0)]])
    out = oracle.unsharded(X, W, None, np.array([0]))
    p = np.array([1 / 6, 1 / 3, 1 / 2])
    dz = p - np.array([1.0, 0, 0])
    assert np.allclose(out["dW"], np.outer(dz, X[0]), atol=1e-15)
    assert np.allclose(out["dX"][0], dz @ W, atol=1e-15)


# P3 -- two classes reduce to logistic regression.
def test_two_class_is_logistic():
    X, W, b, y = _rand_problem(3, 17, 4, 2)
    out = oracle.unsharded(X, W, b, y)
    for i in range(17):
        z = [float(X[i] @ W[c] + b[c]) for c in range(2)]
        d = z[1 - y[i]] - z[y[i]]
        softplus = max(d, 0.0) + math.log1p(math.exp(-abs(d)))
        assert abs(out["loss"][i] - softplus) < 1e-12
        sig = 1.0 / (1.0 + math.exp(-d))          # probability of the wrong class
        assert abs(out["dZ"][i, 1 - y[i]] - sig) < 1e-12
        assert abs(out["dZ"][i, y[i]] + sig) < 1e-12


# P4 -- invariants.
def test_gradient_invariants():
    X, W, b, y = _rand_problem(4, 9, 6, 11)
    out = oracle.unsharded(X, W, b, y)
    assert np.allclose(out["dZ"].sum(axis=1), 0.0, atol=1e-14)
    assert abs(out["db"].sum()) < 1e-13
    assert np.allclose(out["dW"].sum(axis=0), 0.0, atol=1e-13)
    # adding a constant to every bias changes nothing
    out2 = oracle.unsharded(X, W, b + 3.25, y)
    assert np.allclose(out2["loss"], out["loss"], atol=1e-12)
    assert np.allclose(out2["dW"], out["dW"], atol=1e-12)
    assert np.allclose(out2["lse"], out["lse"] + 3.25, atol=1e-12)
    # all class rows equal -> dX = 0
    Weq = np.tile(W[:1], (11, 1))
    assert np.allclose(oracle.unsharded(X, Weq, b, y)["dX"], 0.0, atol=1e-13)
    # linear in g
    out3 = oracle.unsharded(X, W, b, y, g=0.125)
    for k in ("dZ", "dX", "dW", "db"):
        assert np.allclose(out3[k], 0.125 * out[k], rtol=1e-14, atol=0)
    assert np.allclose(out3["loss"], out["loss"])
    assert abs(out["loss_mean"] - sum(out["loss"]) / 9) < 1e-14


# P5 -- partition invariance (Section 2.1: the concatenation of the slice matmuls is the product).
@pytest.mark.parametrize("widths", [[13], [7, 6], [1, 1, 11], [1] * 13, [5, 3, 4, 1], [12, 1]])
def test_partition_invariance(widths):
    B, D, C = 10, 5, 13
    X, W, b, y = _rand_problem(5, B, D, C, scale=2.0)
    full = oracle.unsharded(X, W, b, y, g=0.5)
    ms, ss, ts, offs = [], [], [], []
    o = 0
    hits = np.zeros(B, dtype=int)
    for w in widths:
        m, s, t = oracle.partials(X, W[o:o + w], b[o:o + w], y, o)
        inside, local = oracle.membership(y, o, w)
        hits += inside
        assert np.array_equal(local[inside], y[inside] - o)
        assert np.all(t[~inside] == 0.0)
        ms.append(m), ss.append(s), ts.append(t), offs.append(o)
        o += w
    assert np.array_equal(hits, np.ones(B, dtype=int))          # exactly one shard owns each label
    lse, loss = oracle.combine(ms, ss, ts)
    assert np.allclose(lse, full["lse"], rtol=1e-12, atol=0)
    assert np.allclose(loss, full["loss"], rtol=1e-12, atol=1e-13)
    # row max over shards is the unsharded max and the label logit the unsharded one
    # (to BLAS rounding: a slice matmul may sum in another order than the full one)
    Z = oracle.logits(X, W, b)
    assert np.allclose(np.max(np.stack(ms), axis=0), Z.max(axis=1), rtol=1e-13, atol=1e-14)
    assert np.allclose(np.sum(np.stack(ts), axis=0), Z[np.arange(B), y], rtol=1e-13, atol=1e-14)
    dX = np.zeros((B, D))
    for o, w in zip(offs, widths):
        g = oracle.shard_grads(X, W[o:o + w], b[o:o + w], lse, y, o, g=0.5)
        assert np.allclose(g["dW"], full["dW"][o:o + w], rtol=1e-11, atol=1e-13)
        assert np.allclose(g["db"], full["db"][o:o + w], rtol=1e-11, atol=1e-13)
        assert np.allclose(g["dZ"], full["dZ"][:, o:o + w], rtol=1e-11, atol=1e-14)
        dX += g["dX_partial"]
    assert np.allclose(dX, full["dX"], rtol=1e-11, atol=1e-13)


# P6 -- central finite differences of the summed loss.
def test_finite_differences():
    B, D, C = 3, 4, 5
    X, W, b, y = _rand_problem(6, B, D, C)
    out = oracle.unsharded(X, W, b, y)
    h = 1e-6

    def total(Xv, Wv, bv):
        return float(oracle.unsharded(Xv, Wv, bv, y)["loss"].sum())

    for arr, key in ((X, "dX"), (W, "dW"), (b, "db")):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            save = arr[idx]
            arr[idx] = save + h
            fp = total(X, W, b)
            arr[idx] = save - h
            fm = total(X, W, b)
            arr[idx] = save
            num[idx] = (fp - fm) / (2 * h)
        assert np.allclose(num, out[key], rtol=1e-6, atol=1e-8), key


# P7 -- a library routine for the log-sum-exp special case.
def test_against_scipy_logsumexp():
    X, W, b, y = _rand_problem(7, 12, 8, 40, scale=3.0)
    Z = X @ W.T + b
    out = oracle.unsharded(X, W, b, y)
    assert np.allclose(out["lse"], scipy.special.logsumexp(Z, axis=1), rtol=1e-13)
    assert np.allclose(out["dZ"] + np.eye(40)[y], scipy.special.softmax(Z, axis=1), rtol=1e-11, atol=1e-15)


# P8 -- pure-Python loops on tiny inputs.
@pytest.mark.parametrize("seed,B,D,C", [(8, 4, 3, 6), (9, 8, 8, 16), (10, 1, 1, 1)])
def test_brute_force_loops(seed, B, D, C):
    X, W, b, y = _rand_problem(seed, B, D, C)
    out = oracle.unsharded(X, W, b, y, g=1.5)
    lse, loss, dX, dW, db = tiny_loops.forward_backward(X.tolist(), W.tolist(), b.tolist(), y.tolist(), g=1.5)
    assert np.allclose(out["lse"], lse, rtol=1e-13)
    assert np.allclose(out["loss"], loss, rtol=1e-12, atol=1e-13)
    assert np.allclose(out["dX"], dX, rtol=1e-12, atol=1e-13)
    assert np.allclose(out["dW"], dW, rtol=1e-12, atol=1e-13)
    assert np.allclose(out["db"], db, rtol=1e-12, atol=1e-13)
    if C >= 3:
        lo, hi = 1, C - 1
        m, s, t = oracle.partials(X, W[lo:hi], b[lo:hi], y, lo)
        m2, s2, t2 = tiny_loops.shard_partials(X.tolist(), W.tolist(), b.tolist(), y.tolist(), lo, hi)
        assert np.allclose(m, m2, rtol=1e-13) and np.allclose(s, s2, rtol=1e-13)
        assert np.allclose(t, t2, rtol=1e-13, atol=0)


# P9 -- the integer part: membership and local index, read through the outputs.
def test_membership_through_outputs():
    B, D, C = 64, 2, 50
    r = RNG(11)
    y = r.integers(0, C, size=B)
    X = r.standard_normal((B, D))
    W = np.zeros((C, D))
    b = np.arange(C, dtype=np.float64)
    owners = np.zeros(B, dtype=int)
    for o, w in [(0, 7), (7, 1), (8, 30), (38, 12)]:
        m, s, t = oracle.partials(X, W[o:o + w], b[o:o + w], y, o)
        inside = (y >= o) & (y < o + w)
        assert np.array_equal(t, np.where(inside, y.astype(np.float64), 0.0))
        owners += inside
        # W = 0, b = 0: db recovers the label histogram
        g = oracle.shard_grads(X, W[o:o + w], None, np.full(B, math.log(C)), y, o)
        hist = np.bincount(y[inside] - o, minlength=w)
        assert np.allclose(g["db"], B / C - hist, atol=1e-12)
    assert np.array_equal(owners, np.ones(B, dtype=int))
    # boundary labels
    ins, loc = oracle.membership(np.array([4, 5, 9, 10]), 5, 5)
    assert ins.tolist() == [False, True, True, False]
    assert loc.tolist()[1:3] == [0, 4]


# P10 -- asymptotes and overflow safety.
def test_dominant_logit_and_large_magnitudes():
    C = 6
    X = np.array([[1.0]])
    W = np.zeros((C, 1))
    W[2, 0] = 800.0                      # exp(800) overflows without the max shift
    at_label = oracle.unsharded(X, W, None, np.array([2]))
    assert np.isfinite(at_label["lse"][0]) and abs(at_label["lse"][0] - 800.0) < 1e-12
    assert abs(at_label["loss"][0]) < 1e-12 and np.allclose(at_label["dZ"], 0.0, atol=1e-12)
    off_label = oracle.unsharded(X, W, None, np.array([0]))
    assert abs(off_label["loss"][0] - 800.0) < 1e-9
    assert np.allclose(off_label["dZ"][0], [-1, 0, 1, 0, 0, 0], atol=1e-12)
    # very negative logits must not underflow to log(0)
    out = oracle.unsharded(X, -W - 900.0 * (np.arange(C)[:, None] != 2), None, np.array([1]))
    assert np.all(np.isfinite(out["lse"])) and np.all(np.isfinite(out["loss"]))
    # shard-wise statistics stay finite too, and combine to the same thing
    parts = [oracle.partials(X, W[o:o + 3], None, np.array([0]), o) for o in (0, 3)]
    lse, loss = oracle.combine(*zip(*parts))
    assert abs(lse[0] - 800.0) < 1e-12 and abs(loss[0] - 800.0) < 1e-9


def test_chunked_equals_unchunked():
    X, W, b, y = _rand_problem(12, 37, 6, 19)
    a = oracle.unsharded(X, W, b, y, g=0.3)
    c = oracle.unsharded_chunked(X, W, b, y, g=0.3, rows_per_chunk=8)
    for k in ("lse", "loss", "dX", "dW", "db"):
        assert np.allclose(a[k], c[k], rtol=1e-12, atol=1e-13), k
    # leaving the [C, D] product out changes nothing else
    n = oracle.unsharded_chunked(X, W, b, y, g=0.3, rows_per_chunk=5, want_dW=False)
    assert n["dW"] is None and oracle.unsharded(X, W, b, y, g=0.3, want_dW=False)["dW"] is None
    for k in ("lse", "loss", "dX", "db"):
        assert np.allclose(a[k], n[k], rtol=1e-12, atol=1e-13), k


def test_paper_sizes_fixture():
    """The sizes the paper prints fix D = 2048, C = 100 000, fp32, with a bias."""
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    C = int(vals["classes"])
    fc_mib = (2048 * C + C) * 4 / 2**20
    assert round(fc_mib) == vals["fc_param_mb"]
    assert round(2048 * C * 4 / 2**20) != vals["fc_param_mb"]         # without the bias it would print 781
    share = vals["fc_param_mb"] / (vals["fc_param_mb"] + vals["resnet50_param_mb"])
    assert round(100 * share, 1) == vals["sync_reduction_percent"]


# ---- predictions = Softmax(logits) per shard (the split listing of Section 3.1.2) -----------------

def test_predictions_hand_example_and_row_sums():
    # the three-class example above: softmax = (1/6, 1/3, 1/2); shards (2 classes, 1 class)
    X = np.array([[1.0]]); W = np.array([[0.0], [math.log(2.0)], [math.log(3.0)]])
    lse = np.array([math.log(6.0)])
    assert np.allclose(oracle.predictions(X, W[:2], None, lse), [[1 / 6, 1 / 3]], rtol=1e-15)
    assert np.allclose(oracle.predictions(X, W[2:], None, lse), [[1 / 2]], rtol=1e-15)


def test_predictions_concatenate_to_the_softmax():
    rng = np.random.default_rng(12)
    B, D, C = 9, 7, 23
    X = rng.normal(size=(B, D)); W = rng.normal(size=(C, D)); b = rng.normal(size=C)
    y = rng.integers(0, C, size=B)
    ref = oracle.unsharded(X, W, b, y, 1.0)
    shards = [(0, 1), (1, 15), (16, 7)]
    P = np.concatenate([oracle.predictions(X, W[o:o + c], b[o:o + c], ref["lse"]) for o, c in shards], axis=1)
    assert np.allclose(P, scipy.special.softmax(oracle.logits(X, W, b), axis=1), rtol=1e-12, atol=1e-15)
    assert np.allclose(P.sum(axis=1), 1.0, rtol=1e-13)
    onehot = np.zeros((B, C)); onehot[np.arange(B), y] = 1.0
    assert np.allclose(P - onehot, ref["dZ"], rtol=1e-12, atol=1e-15)      # dz = softmax - onehot at g = 1
    # with a shard's own log-sum-exp instead of the combined one the rows would not sum to 1:
    m, s, _ = oracle.partials(X, W[:16], b[:16], y, 0)
    own = oracle.predictions(X, W[:16], b[:16], m + np.log(s))
    assert np.allclose(own.sum(axis=1), 1.0) and not np.allclose(P[:, :16].sum(axis=1), 1.0)


# ---- the contraction-split sharding pattern (SP2 of Section 3.2.2) -------------------------------

def test_sp2_hand_example():
    X = np.array([[1.0, 2.0]]); W = np.array([[3.0, 4.0], [5.0, 6.0]])
    assert oracle.sp2_partial_logits(X, W, 0, 1).tolist() == [[3.0, 5.0]]
    assert oracle.sp2_partial_logits(X, W, 1, 2).tolist() == [[8.0, 12.0]]      # sum = X . W^T = (11, 17)
    lse, loss = oracle.sp2_reduce([np.array([[3.0, 5.0]]), np.array([[8.0, 12.0]])], None, [1])
    assert abs(lse[0] - (17.0 + math.log1p(math.exp(-6.0)))) < 1e-14
    assert abs(loss[0] - math.log1p(math.exp(-6.0))) < 1e-14


def test_sp2_partials_sum_to_the_logits_and_give_the_same_loss():
    rng = np.random.default_rng(14)
    B, D, C = 7, 12, 19
    X = rng.normal(size=(B, D)); W = rng.normal(size=(C, D)); b = rng.normal(size=C)
    y = rng.integers(0, C, size=B)
    ref = oracle.unsharded(X, W, b, y, 1.0)
    for cuts in ([0, 12], [0, 1, 12], [0, 4, 8, 12], list(range(13))):
        parts = [oracle.sp2_partial_logits(X, W, a, e) for a, e in zip(cuts[:-1], cuts[1:])]
        assert all(p.shape == (B, C) for p in parts)          # every slice yields ALL classes
        assert np.allclose(sum(parts), oracle.logits(X, W, None), rtol=1e-12, atol=1e-13)
        lse, loss = oracle.sp2_reduce(parts, b, y)
        assert np.allclose(lse, ref["lse"], rtol=1e-13) and np.allclose(loss, ref["loss"], rtol=1e-11, atol=1e-13)


# ---- the weight update that ends a mini-batch (Section 2.1) ----------------------------------------

def test_sgd_update_descends_by_the_squared_gradient_norm():
    """First-order Taylor: loss(theta - lr * grad) = loss(theta) - lr * |grad|^2 + O(lr^2).  A wrong sign, a
    missing factor or swapped gradients fail this."""
    rng = np.random.default_rng(15)
    B, D, C = 6, 5, 7
    X = rng.normal(size=(B, D)); W = rng.normal(size=(C, D)); b = rng.normal(size=C)
    y = rng.integers(0, C, size=B)
    ref = oracle.unsharded(X, W, b, y, 1.0)
    g2 = float((ref["dW"] ** 2).sum() + (ref["db"] ** 2).sum())
    for lr in (1e-4, 1e-5):
        Wn, bn = oracle.sgd_update(W, b, ref["dW"], ref["db"], lr)
        after = oracle.unsharded(X, Wn, bn, y, 1.0)["loss"].sum()
        drop = ref["loss"].sum() - after
        assert abs(drop - lr * g2) <= 50 * lr * lr * g2 + 1e-13
    Wn, bn = oracle.sgd_update(W, b, ref["dW"], ref["db"], 0.0)
    assert np.array_equal(Wn, W) and np.array_equal(bn, b)
    Wn, bn = oracle.sgd_update(W, None, ref["dW"], None, 0.5)
    assert bn is None and np.allclose(Wn, W - 0.5 * ref["dW"], rtol=0, atol=0)


# ---- arg-max predictions and their merge across shards ------------------------------------------------

def test_top1_hand_example_ties_and_merge():
    X = np.array([[1.0], [-1.0]]); W = np.array([[0.0], [2.0], [2.0], [-3.0]])
    v, c = oracle.top1(X, W, None, 0)
    assert v.tolist() == [2.0, 3.0] and c.tolist() == [1, 3]        # row 0: classes 1 and 2 tie -> the lower id
    v0, c0 = oracle.top1(X, W[:2], None, 0)
    v1, c1 = oracle.top1(X, W[2:], None, 2)
    assert c0.tolist() == [1, 0] and c1.tolist() == [2, 3]
    bv, bc = oracle.combine_top1([v0, v1], [c0, c1])
    assert bv.tolist() == [2.0, 3.0] and bc.tolist() == [1, 3]      # the tie across shards also goes to the lower id


def test_top1_merge_equals_argmax_of_the_whole_layer():
    rng = np.random.default_rng(16)
    X = rng.normal(size=(40, 6)); W = rng.normal(size=(37, 6)); b = rng.normal(size=37)
    Z = oracle.logits(X, W, b)
    parts = [oracle.top1(X, W[o:o + c], b[o:o + c], o) for o, c in [(0, 1), (1, 20), (21, 16)]]
    bv, bc = oracle.combine_top1([p[0] for p in parts], [p[1] for p in parts])
    assert np.array_equal(bc, Z.argmax(axis=1)) and np.array_equal(bv, Z.max(axis=1))
    # the arg-max of the logits is the arg-max of the softmax (monotone), so these are the predictions
    assert np.array_equal(bc, scipy.special.softmax(Z, axis=1).argmax(axis=1))
