"""GPU parity of the bridge-layer ends (Section 3.2.3) through the C-ABI binding: the gather is byte
work and must be bit-exact; the reduce is an fp32 sum in a fixed order, checked bit for bit against
the same sum in numpy float32 and against the fp64 oracle within the rounding bound of S terms."""
import numpy as np
import pytest

from oracle import bridge as ob
from paper_2011_09208_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU fallback")
    return torch


@pytest.fixture(scope="module")
def ws():
    from paper_2011_09208_amd import binding
    return binding


def say(msg):
    print(msg, flush=True)


def _gather_case(T, ws, dim, extents, other, np_dtype, pad_in=0, pad_out=0, shift=0, seed=0):
    """Parts are views into larger buffers (pitch = width + pad_in, first element `shift` elements in)."""
    rng = np.random.default_rng(seed)
    tdt = {np.uint16: T.int16, np.uint32: T.int32}[np_dtype]
    host, dev = [], []
    for e in extents:
        shape = (e, other) if dim == 0 else (other, e)
        a = rng.integers(0, np.iinfo(np_dtype).max, size=shape, dtype=np_dtype)
        host.append(a)
        buf = T.full((shape[0] * (shape[1] + pad_in) + shift + 8,), -1, dtype=tdt, device="cuda")
        view = buf[shift: shift + shape[0] * (shape[1] + pad_in)].view(shape[0], shape[1] + pad_in)[:, :shape[1]]
        view.copy_(T.from_numpy(a.view(np.int16 if np_dtype == np.uint16 else np.int32)).cuda())
        dev.append(view)
    total = sum(extents)
    oshape = (total, other) if dim == 0 else (other, total)
    obuf = T.full((oshape[0], oshape[1] + pad_out), -1, dtype=tdt, device="cuda")
    out = obuf[:, :oshape[1]]
    ws.bridge_gather(dim, dev, out)
    T.cuda.synchronize()
    got = obuf.cpu().numpy().view(np_dtype)
    ref = ob.gather(dim, host)
    assert np.array_equal(got[:, :oshape[1]], ref)
    if pad_out:
        assert np.all(got[:, oshape[1]:] == np.iinfo(np_dtype).max)     # padding columns untouched (-1)


def test_gather_replicate_pattern_features(T, ws):
    say("[bridge] gather dim 0: 8 replicas x 128 rows x 2048 bf16 (the paper's shape at B = 1024)")
    _gather_case(T, ws, 0, [128] * 8, 2048, np.uint16)
    say("[bridge] gather dim 0: uneven batches incl. an empty replica, padded pitches")
    _gather_case(T, ws, 0, [37, 0, 201, 1, 90], 2048, np.uint16, pad_in=8, pad_out=16, seed=1)
    say("[bridge] gather dim 0: narrow rows (packed several per workgroup), fp32")
    _gather_case(T, ws, 0, [1000, 3, 517], 12, np.uint32, seed=2)


def test_gather_split_pattern_columns(T, ws):
    say("[bridge] gather dim 1: uneven shard widths, 16-byte path")
    _gather_case(T, ws, 1, [376, 128, 376, 128], 64, np.uint16, seed=3)
    say("[bridge] gather dim 1: odd widths force the 2-byte path")
    _gather_case(T, ws, 1, [5, 1, 0, 7, 3], 33, np.uint16, pad_in=3, pad_out=1, seed=4)
    say("[bridge] gather dim 1: fp32, 4- and 8-byte paths")
    _gather_case(T, ws, 1, [3, 9, 5], 19, np.uint32, seed=5)
    _gather_case(T, ws, 1, [6, 10, 2], 19, np.uint32, pad_in=2, pad_out=2, seed=6)


def test_gather_misaligned_bases(T, ws):
    say("[bridge] gather dim 0: part bases 2 bytes off a 16-byte boundary")
    _gather_case(T, ws, 0, [9, 17], 64, np.uint16, shift=1, seed=7)
    _gather_case(T, ws, 0, [9, 17], 64, np.uint16, shift=4, seed=8)     # 8-byte aligned
    say("[bridge] gather: the maximum number of parts")
    _gather_case(T, ws, 0, [3] * 64, 40, np.uint16, seed=9)


def _reduce_case(T, ws, S, rows, D, pad=0, seed=0):
    rng = np.random.default_rng(seed)
    B = sum(rows)
    parts_h = [(rng.standard_normal((B, D)) * 10.0 ** rng.integers(-3, 3)).astype(np.float32) for _ in range(S)]
    parts_d = []
    for a in parts_h:
        buf = T.full((B, D + pad), float("nan"), device="cuda")
        buf[:, :D].copy_(T.from_numpy(a).cuda())
        parts_d.append(buf[:, :D])
    outs_b = [T.full((max(r, 1), D + pad), float("nan"), device="cuda") for r in rows]
    outs = [b[:r, :D] for b, r in zip(outs_b, rows)]
    ws.bridge_reduce_partition(parts_d, outs)
    T.cuda.synchronize()
    got = [o.cpu().numpy() for o in outs]
    # (1) same precision, same order: bit for bit
    acc = parts_h[0].copy()
    for a in parts_h[1:]:
        acc = acc + a
    at = 0
    for g, r in zip(got, rows):
        assert g.shape == (r, D)
        assert np.array_equal(g, acc[at:at + r])
        at += r
    # (2) the fp64 oracle within the rounding bound of S - 1 fp32 additions
    ref = ob.reduce_partition(parts_h, rows)
    bound = (S - 1) * 2.0 ** -24 * sum(np.abs(a.astype(np.float64)) for a in parts_h) + 1e-45
    at = 0
    for g, rf, r in zip(got, ref, rows):
        assert np.all(np.abs(g - rf) <= bound[at:at + r])
        at += r
    if pad:
        for b in outs_b:
            assert bool(T.isnan(b[:, D:]).all())


def test_reduce_partition(T, ws):
    say("[bridge] reduce+partition: 8 shards, 8 replicas x 128 rows x 2048 (the paper's shape)")
    _reduce_case(T, ws, 8, [128] * 8, 2048)
    say("[bridge] reduce+partition: uneven rows incl. an empty replica, padded pitches, one shard")
    _reduce_case(T, ws, 1, [5, 0, 90, 33], 256, pad=4, seed=1)
    say("[bridge] reduce+partition: narrow rows, 64 shards")
    _reduce_case(T, ws, 64, [100, 1, 27], 12, seed=2)


def test_bridge_around_the_split_head(T, ws):
    """Features arrive as replica blocks, are gathered into X, go through fwd/bwd of two shards, and the
    shards' dX_partial go back through reduce+partition: every replica gets the oracle's dX rows."""
    from tests import gpu_harness as H
    from oracle import oracle
    p = inputs.make_config("cfg1")
    rows = [5, 16, 0, 11]
    B, D = p.B, p.D
    X_all = H.dev_bf16(p.X_bits)
    blocks, at = [], 0
    for r in rows:
        blocks.append(X_all[at:at + r].clone())
        at += r
    X = T.empty((B, D), dtype=T.bfloat16, device="cuda")
    ws.bridge_gather(0, blocks, X)
    assert T.equal(X.view(T.int16), X_all.view(T.int16))
    W = H.dev_bf16(p.W_bits)
    y = T.from_numpy(p.labels.astype(np.int32)).cuda()
    S = len(p.shards)
    m = T.empty((S, B), device="cuda"); s = T.empty((S, B), device="cuda"); t = T.empty((S, B), device="cuda")
    lse = T.empty(B, device="cuda"); loss = T.empty(B, device="cuda")
    work = T.empty(max(max(ws.fwd_workspace_bytes(B, D, c), ws.bwd_workspace_bytes(B, D, c)) for _, c in p.shards),
                   dtype=T.uint8, device="cuda")
    for i, (off, c) in enumerate(p.shards):
        ws.split_fc_fwd(X, W[off:off + c], None, y, off, m[i], s[i], t[i], work)
    ws.combine_partials(m, s, t, lse, loss, None)
    partials = []
    for i, (off, c) in enumerate(p.shards):
        dXp = T.empty((B, D), device="cuda")
        dW = T.empty((c, D), dtype=T.bfloat16, device="cuda")
        ws.split_fc_bwd(X, W[off:off + c], None, lse, y, off, 1.0, dXp, False, dW, None, work)
        partials.append(dXp)
    outs = [T.full((r, D), float("nan"), device="cuda") for r in rows]
    ws.bridge_reduce_partition(partials, outs)
    T.cuda.synchronize()
    ref = oracle.unsharded(inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits), None,
                           p.labels.astype(np.int64), 1.0)
    ref_parts = ob.partition(ref["dX"], 0, rows)
    scale = np.max(np.abs(ref["dX"]))
    for o, rf in zip(outs, ref_parts):
        assert np.max(np.abs(o.cpu().numpy() - rf), initial=0.0) <= H.GRAD_REL_TO_MAX * scale
