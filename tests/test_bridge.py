"""Bridge-layer ends (Section 3.2.3): pins of the oracle, the host-side fusion rule of the library
against the oracle, and argument validation of the two GPU entry points (no GPU needed)."""
import ctypes

import numpy as np
import pytest

from oracle import bridge as ob
from oracle import oracle
from paper_2011_09208_amd import inputs


@pytest.fixture(scope="module")
def ws():
    from paper_2011_09208_amd import buildlib
    if buildlib.is_stale():
        buildlib.build()
    from paper_2011_09208_amd import binding
    return binding


# ---- oracle pins ------------------------------------------------------------------------------

def test_hand_example_replicate_and_split_patterns():
    # two replicas with 1 and 2 samples: rows stack (batch_dim)
    a = np.array([[1, 2]]); b = np.array([[3, 4], [5, 6]])
    assert ob.gather(0, [a, b]).tolist() == [[1, 2], [3, 4], [5, 6]]
    # two shards with 1 and 2 columns: columns stack (split_dim)
    c = np.array([[1], [2]]); d = np.array([[3, 4], [5, 6]])
    assert ob.gather(1, [c, d]).tolist() == [[1, 3, 4], [2, 5, 6]]


def test_gather_by_element_loops():
    rng = np.random.default_rng(3)
    for dim in (0, 1):
        ext = [3, 0, 5, 1]
        parts = [rng.integers(0, 1000, size=(e, 4) if dim == 0 else (4, e)) for e in ext]
        got = ob.gather(dim, parts)
        at = 0
        for p in parts:                      # every element lands at (its index + the offset of its part)
            for i in range(p.shape[0]):
                for j in range(p.shape[1]):
                    gi, gj = (at + i, j) if dim == 0 else (i, at + j)
                    assert got[gi, gj] == p[i, j]
            at += p.shape[dim]
        assert got.shape[dim] == sum(ext)


def test_partition_inverts_gather():
    rng = np.random.default_rng(4)
    for dim in (0, 1):
        ext = [7, 2, 9]
        parts = [rng.normal(size=(e, 5) if dim == 0 else (5, e)) for e in ext]
        back = ob.partition(ob.gather(dim, parts), dim, ext)
        for p, q in zip(parts, back):
            assert np.array_equal(p, q)


def test_split_pattern_gather_of_logits_is_the_unsharded_product():
    # Section 2.1: the column slices' products concatenate to the full product
    rng = np.random.default_rng(5)
    X = rng.normal(size=(6, 8)); W = rng.normal(size=(11, 8)); b = rng.normal(size=11)
    shards = [(0, 4), (4, 1), (5, 6)]
    parts = [oracle.logits(X, W[o:o + c], b[o:o + c]) for o, c in shards]
    assert np.allclose(ob.gather(1, parts), oracle.logits(X, W, b), rtol=1e-13, atol=1e-13)


def test_reduce_partition_gives_each_replica_its_rows_of_dX():
    # the shards' dX_partial sum to the unsharded dX; the bridge hands replica r its batch rows
    rng = np.random.default_rng(6)
    B, D, C = 10, 8, 13
    X = rng.normal(size=(B, D)); W = rng.normal(size=(C, D)); b = rng.normal(size=C)
    y = rng.integers(0, C, size=B)
    ref = oracle.unsharded(X, W, b, y, 1.0)
    shards = [(0, 5), (5, 8)]
    partials = [oracle.shard_grads(X, W[o:o + c], b[o:o + c], ref["lse"], y, o, 1.0)["dX_partial"] for o, c in shards]
    rows = [3, 0, 6, 1]
    outs = ob.reduce_partition(partials, rows)
    assert [o.shape[0] for o in outs] == rows
    assert np.allclose(np.concatenate(outs, axis=0), ref["dX"], rtol=1e-12, atol=1e-13)
    # replica r's block is the gradient of ITS samples only: it equals the dX of a step on those rows
    at = 3
    sub = oracle.unsharded(X[at:at + 6], W, b, y[at:at + 6], 1.0)
    assert np.allclose(outs[2], sub["dX"], rtol=1e-12, atol=1e-13)


def test_fusion_rule_truth_table():
    assert ob.fusable(0, [4, 4], 0, [4, 4])
    assert not ob.fusable(0, [4, 4], 1, [4, 4])          # other dimension
    assert not ob.fusable(0, [4, 4], 0, [2, 6])          # same dimension, other cuts
    assert not ob.fusable(0, [8], 0, [4, 4])             # other number of parts
    assert ob.fusable(1, [3, 0, 5], 1, [3, 0, 5])
    # when it holds, gather followed by partition is the identity on the parts
    parts = [np.arange(8).reshape(4, 2), np.arange(8, 16).reshape(4, 2)]
    back = ob.partition(ob.gather(0, parts), 0, [4, 4])
    assert all(np.array_equal(p, q) for p, q in zip(parts, back))


# ---- library host code against the oracle -------------------------------------------------------

def test_library_fusion_rule_equals_oracle(ws):
    rng = np.random.default_rng(7)
    for _ in range(300):
        n = int(rng.integers(1, 5))
        src = rng.integers(0, 4, size=n).tolist()
        dst = src.copy() if rng.random() < 0.5 else rng.integers(0, 4, size=int(rng.integers(1, 5))).tolist()
        gd, pd = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        assert ws.bridge_fusable(gd, src, pd, dst) == ob.fusable(gd, src, pd, dst)


A = 0x10000     # fake 16-byte aligned "device" address: validation never dereferences it


def _gather(ws, dim=0, parts=(A, A), lds=(64, 64), ext=(3, 5), n=None, other=64, eb=2, out=A, ld_out=64):
    k = len(parts)
    P = (ctypes.c_void_p * k)(*parts)
    L = (ctypes.c_int64 * k)(*lds)
    E = (ctypes.c_int32 * k)(*ext)
    return ws.lib.ws_bridge_gather(dim, P, L, E, k if n is None else n, other, eb, out, ld_out, None)


def _reduce(ws, parts=(A, A), lds=(64, 64), S=None, D=64, outs=(A, A), ldo=(64, 64), rows=(3, 5), R=None):
    P = (ctypes.c_void_p * len(parts))(*parts)
    L = (ctypes.c_int64 * len(parts))(*lds)
    O = (ctypes.c_void_p * len(outs))(*outs)
    LO = (ctypes.c_int64 * len(outs))(*ldo)
    RW = (ctypes.c_int32 * len(outs))(*rows)
    return ws.lib.ws_bridge_reduce_partition(P, L, len(parts) if S is None else S, D, O, LO, RW,
                                             len(outs) if R is None else R, None)


def test_bridge_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(7)}
    assert ws.lib.ws_bridge_gather(0, None, None, None, 1, 4, 2, A, 4, None) == E["WS_ERR_NULL"]
    assert _gather(ws, dim=2) == E["WS_ERR_RANGE"]
    assert _gather(ws, n=0) == E["WS_ERR_RANGE"]
    assert _gather(ws, parts=(A,) * 65, lds=(64,) * 65, ext=(1,) * 65) == E["WS_ERR_RANGE"]
    assert _gather(ws, eb=3) == E["WS_ERR_SHAPE"]
    assert _gather(ws, other=0) == E["WS_ERR_SHAPE"]
    assert _gather(ws, ext=(3, -1)) == E["WS_ERR_SHAPE"]
    assert _gather(ws, lds=(64, 63)) == E["WS_ERR_SHAPE"]           # pitch below the row length
    assert _gather(ws, ld_out=63) == E["WS_ERR_SHAPE"]
    assert _gather(ws, dim=1, other=4, ext=(3, 5), lds=(3, 5), ld_out=7) == E["WS_ERR_SHAPE"]   # 3 + 5 columns
    assert _gather(ws, parts=(A, None)) == E["WS_ERR_NULL"]
    assert _gather(ws, parts=(A, A + 1)) == E["WS_ERR_ALIGN"]
    assert _gather(ws, eb=4, parts=(A, A + 2)) == E["WS_ERR_ALIGN"]
    assert _gather(ws, ext=(0, 0)) == E["WS_OK"]                    # nothing to copy: no launch

    assert _reduce(ws, S=0) == E["WS_ERR_RANGE"]
    assert _reduce(ws, R=65) == E["WS_ERR_RANGE"]
    assert _reduce(ws, D=66) == E["WS_ERR_SHAPE"]
    assert _reduce(ws, lds=(64, 60)) == E["WS_ERR_SHAPE"]
    assert _reduce(ws, ldo=(60, 64)) == E["WS_ERR_SHAPE"]
    assert _reduce(ws, rows=(3, -5)) == E["WS_ERR_SHAPE"]
    assert _reduce(ws, parts=(A, A + 4)) == E["WS_ERR_ALIGN"]
    assert _reduce(ws, outs=(A + 8, A)) == E["WS_ERR_ALIGN"]
    assert _reduce(ws, lds=(66, 64)) == E["WS_ERR_ALIGN"]
    assert _reduce(ws, parts=(A, None)) == E["WS_ERR_NULL"]
    assert _reduce(ws, rows=(0, 0)) == E["WS_OK"]

    ok = ctypes.c_int32(0)
    a = (ctypes.c_int64 * 2)(1, 2)
    assert ws.lib.ws_bridge_fusable(0, 2, a, 0, 2, None, ctypes.byref(ok)) == E["WS_ERR_NULL"]
    assert ws.lib.ws_bridge_fusable(0, 0, a, 0, 2, a, ctypes.byref(ok)) == E["WS_ERR_RANGE"]
    assert ws.lib.ws_bridge_fusable(-1, 2, a, 0, 2, a, ctypes.byref(ok)) == E["WS_ERR_RANGE"]
    neg = (ctypes.c_int64 * 2)(1, -2)
    assert ws.lib.ws_bridge_fusable(0, 2, neg, 0, 2, a, ctypes.byref(ok)) == E["WS_ERR_SHAPE"]
