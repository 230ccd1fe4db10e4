"""GPU parity: the HIP path, called through the C-ABI binding, against the fp64 oracle on the
same seeded bf16 inputs.  Gate: loss rel <= 1e-3, logsumexp abs <= 2e-3, every gradient
<= 2e-2 * max|grad| in max-abs, label/shard membership bit-exact.  The workload configurations
are held to exactly these figures; gpu_harness.compare documents the two wider variants used
for random ragged shapes (an fp32 rounding floor on per-row losses near zero) and for the
large-logit stress cases (absolute gates scaled by |z|max)."""
import math

import numpy as np
import pytest

from paper_2011_09208_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU fallback")
    from tests import gpu_harness
    return gpu_harness


def _full_parity(H, p, shards, g=1.0, tag="", gate="fp32_floor", **kw):
    shape = f"B={p.B} D={p.D} C={p.C} shards={shards if len(shards) < 6 else len(shards)} g={g:.3g}"
    H.say(f"[parity] {tag}: {shape}")
    got = H.run_step(p.X_bits, p.W_bits, p.bias, p.labels, shards, g=g, w_lo=p.w_lo, **kw)
    ref = H.oracle_step(p.X_bits, p.W_bits, p.bias, p.labels, shards, g=g, w_lo=p.w_lo)
    rep = H.compare(got, ref, p.labels, shards, tag, gate=gate)
    H.say(f"[parity] {tag}: " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()))
    H.record(tag, f"{shape} gate={gate}", rep)
    return got, ref


def test_cfg1_tiny(H):
    p = inputs.make_config("cfg1")
    got, ref = _full_parity(H, p, p.shards, tag="cfg1", gate="stated", loss_mean=True)
    assert abs(got["loss_mean"] - ref["loss"].mean()) <= 1e-3 * ref["loss"].mean()
    # near-uniform logits: the loss sits next to ln C
    assert abs(ref["loss"].mean() - math.log(1000)) < 0.05


@pytest.mark.parametrize("B,D,widths", [
    (1, 64, [1]),
    (37, 192, [127, 129, 1, 128]),
    (300, 256, [500, 700, 77]),
    (257, 64, [255, 257, 256]),
    (513, 128, [1030]),
    (300, 4096, [600]),
    (5000, 64, [40, 7]),
])
def test_ragged_shapes_with_bias(H, B, D, widths):
    """Row counts and shard widths that are not multiples of any tile, several tiles wide, with a
    non-zero bias (exercises the recompute's bias path) and the mean-loss gradient scale."""
    C = sum(widths)
    p = inputs.make_inputs("ragged", B, D, C, x_sigma=1.0, w_sigma=0.2, bias_sigma=1.0, seed=B + D)
    shards, o = [], 0
    for w in widths:
        shards.append((o, w))
        o += w
    _full_parity(H, p, shards, g=1.0 / B, tag=f"ragged B={B} D={D} widths={widths}")


# Shapes chosen by how the launch is cut into tiles (a tile is 256 classes x 256 rows; a launch of at most 128
# tiles, or the last partial round of a longer one when it fills at most half of the 256 compute units, runs
# as four 256 x 64 "thin" tiles per tile).  The shapes above all have fewer than 128 tiles, i.e. only thin ones.
FULL_TILES_RAGGED = dict(B=300, D=64, C=256 * 70 + 5)      # 2 x 71 = 142 tiles: all full; ragged batch and class edge
MIXED_TILES_RAGGED = dict(B=513, D=64, C=256 * 90 + 17)    # 3 x 91 = 273 tiles: 256 full + 17 x 4 thin, ragged edges
MIXED_FIVE_BATCH_TILES = dict(B=1100, D=128, C=14000)      # 5 x 55 = 275 tiles: 256 full + 19 x 4 thin
# the dW kernel tiles features x classes: 4 x 71 = 284 tiles, more than one round of the 256 compute units
MIXED_DW_TILES = dict(B=300, D=1024, C=256 * 70 + 5)
# long contractions in the dW kernel (B >= 3072 rows: 48 k-steps), where it cuts a ragged last round into thin
# tiles too; 13 batch tiles (logits tiles numbered in blocks of 8 class x 4 batch tiles, the last block 1 wide)
LONG_K_DW_ALL_THIN = dict(B=3100, D=320, C=600)              # dW: 2 x 3 = 6 tiles, all thin; ragged feature tile
LONG_K_DW_MIXED = dict(B=3100, D=2304, C=256 * 29 - 7)       # dW: 9 x 29 = 261 tiles: 256 full + 5 x 4 thin


@pytest.mark.parametrize("shape,g", [
    (FULL_TILES_RAGGED, 1.0 / 300),
    (FULL_TILES_RAGGED, -0.75),
    (MIXED_TILES_RAGGED, 1.0 / 513),
    (MIXED_TILES_RAGGED, -2.0 / 513),
    (MIXED_FIVE_BATCH_TILES, 1.0 / 1100),
    (MIXED_DW_TILES, 1.0 / 300),
    (LONG_K_DW_ALL_THIN, 1.0 / 3100),
    (LONG_K_DW_MIXED, -3.0 / 3100),
], ids=["full-tiles", "full-tiles-negative-scale", "mixed-tiles", "mixed-tiles-negative-scale", "mixed-5-batch-tiles",
        "mixed-dw-tiles", "long-k-dw-thin-tiles", "long-k-dw-mixed-tiles-negative-scale"])
def test_full_and_mixed_tile_launches_ragged_with_bias(H, shape, g):
    """The full-tile epilogues of the forward and dz kernels with everything the small shapes only reach on
    thin tiles: a batch edge inside a tile, a class edge inside a tile, a non-zero bias, a fractional and a
    negative gradient scale; and launches that mix full and thin tiles at those edges."""
    B, D, C = shape["B"], shape["D"], shape["C"]
    p = inputs.make_inputs("tiles", B, D, C, x_sigma=1.0, w_sigma=0.25, bias_sigma=1.0, seed=B + C)
    _full_parity(H, p, [(0, C)], g=g, tag=f"tiles B={B} D={D} C={C} g={g:.3g}")


def test_full_and_mixed_tile_launches_two_shards(H):
    """The mixed launch shape again as the second of two uneven shards (non-zero class offset, labels on
    both sides of the cut), so that membership and the one-hot term are exercised on full tiles too."""
    B, D = 513, 64
    widths = [777, 256 * 90 + 17]
    C = sum(widths)
    p = inputs.make_inputs("tiles2", B, D, C, x_sigma=1.0, w_sigma=0.25, bias_sigma=1.0, seed=77)
    _full_parity(H, p, [(0, widths[0]), (widths[0], widths[1])], g=1.0 / B, tag=f"tiles two shards B={B} widths={widths}")


def _random_shapes(n, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(n):
        B = int(r.integers(1, 1400))
        D = 64 * int(r.integers(1, 9))
        n_shards = int(r.integers(1, 4))
        widths = [int(w) for w in r.integers(1, 12000, size=n_shards)]
        g = float(r.choice([1.0, 1.0 / B, -0.5, 3.0]))
        out.append((B, D, widths, g, bool(r.integers(0, 2)), int(r.integers(0, 1 << 30))))
    return out


@pytest.mark.parametrize("B,D,widths,g,with_bias,seed", _random_shapes(10, 2024),
                         ids=lambda v: str(v) if not isinstance(v, list) else "x".join(map(str, v)))
def test_seeded_random_shapes(H, B, D, widths, g, with_bias, seed):
    """Ten seeded random problems (row count, feature count, one to three uneven shards, gradient scale,
    bias on or off): whatever mix of full tiles, thin tiles, ragged edges and split-K ranges they produce."""
    C = sum(widths)
    p = inputs.make_inputs("random", B, D, C, x_sigma=1.0, w_sigma=0.3, bias_sigma=1.0 if with_bias else None, seed=seed)
    shards, o = [], 0
    for w in widths:
        shards.append((o, w))
        o += w
    _full_parity(H, p, shards, g=g, tag=f"random B={B} D={D} widths={widths}")


def test_large_logits_and_dominant_class(H):
    """|z| of a few hundred: a missing max-subtraction overflows fp32; a planted dominant logit at the
    label drives loss and dz to ~0, at another class the loss equals the gap."""
    B, D, C = 96, 128, 640
    p = inputs.make_inputs("large", B, D, C, x_sigma=1.0, w_sigma=1.5, seed=5)
    W = inputs.bf16_bits_to_f32(p.W_bits).copy()
    X = inputs.bf16_bits_to_f32(p.X_bits)
    y = p.labels.copy()
    # rows 0..31: make the label's class row a large multiple of the sample itself
    for i in range(16):
        y[i] = 40 + i                     # distinct classes so the planted rows do not collide
        W[y[i]] = 2.0 * X[i]
    for i in range(16, 32):
        y[i] = 100 + i
        W[300 + i] = 2.0 * X[i]           # dominant logit at a class that is not the label
    p.W_bits = inputs.f32_to_bf16_bits(W)
    p.labels = y
    shards = [(0, 200), (200, 300), (500, 140)]
    got, ref = _full_parity(H, p, shards, tag="large-logits", gate="large_logits")
    assert np.max(np.abs(ref["m"])) > 100.0
    assert np.all(ref["loss"][:16] < 1e-6) and np.all(np.abs(got["loss"][:16]) < 1e-3)
    assert np.all(ref["loss"][16:32] > 50.0)


def test_membership_is_bit_exact(H):
    """W = 0 and b_c = c make every logit an exactly representable integer, so label_logit must be
    exactly float(label) inside the shard and exactly 0 outside; with b = 0, db recovers the label
    histogram of the shard."""
    B, D, C = 700, 64, 1500
    p = inputs.make_inputs("member", B, D, C, seed=9)
    p.W_bits = np.zeros_like(p.W_bits)
    shards = [(0, 1), (1, 255), (256, 256), (512, 513), (1025, 475)]
    y = p.labels.copy()
    y[:10] = [0, 1, 255, 256, 511, 512, 1024, 1025, 1499, 1]      # shard boundaries
    p.labels = y
    bias = np.arange(C, dtype=np.float32)
    H.say("[parity] membership: label_logit with b_c = c")
    got = H.run_step(p.X_bits, p.W_bits, bias, y, shards)
    owners = np.zeros(B, dtype=int)
    for i, (off, c) in enumerate(shards):
        inside = (y >= off) & (y < off + c)
        owners += inside
        assert np.array_equal(got["t"][i], np.where(inside, y.astype(np.float32), np.float32(0.0)))
        assert np.array_equal(got["m"][i], np.full(B, np.float32(off + c - 1)))
    assert np.array_equal(owners, np.ones(B, dtype=int))
    H.say("[parity] membership: db histogram with b = 0")
    got = H.run_step(p.X_bits, p.W_bits, None, y, shards)
    assert np.allclose(got["lse"], math.log(C), atol=1e-5)
    for i, (off, c) in enumerate(shards):
        inside = (y >= off) & (y < off + c)
        hist = np.bincount(y[inside] - off, minlength=c)
        recovered = np.rint(B / C - got["db"][i].astype(np.float64)).astype(np.int64)
        assert np.array_equal(recovered, hist)
        assert np.max(np.abs(got["db"][i] - (B / C - hist))) < 5e-2


def test_all_or_no_labels_in_shard(H):
    B, D, C = 130, 64, 900
    p = inputs.make_inputs("allnone", B, D, C, w_sigma=0.3, seed=3)
    p.labels = (p.labels % 300 + 300).astype(np.int32)            # every label inside the middle shard
    shards = [(0, 300), (300, 300), (600, 300)]
    got, ref = _full_parity(H, p, shards, tag="all-or-none")
    assert np.all(got["t"][0] == 0.0) and np.all(got["t"][2] == 0.0)


def test_run_twice_bit_identical(H):
    p = inputs.make_inputs("twice", 300, 128, 1000, w_sigma=0.3, bias_sigma=0.5, seed=2)
    shards = [(0, 600), (600, 400)]
    H.say("[parity] determinism: two runs of the same step")
    a = H.run_step(p.X_bits, p.W_bits, p.bias, p.labels, shards)
    b = H.run_step(p.X_bits, p.W_bits, p.bias, p.labels, shards)
    for k in ("m", "s", "t", "lse", "loss", "dX"):
        assert np.array_equal(a[k], b[k]), k
    for i in range(2):
        assert np.array_equal(a["dW"][i], b["dW"][i]) and np.array_equal(a["db"][i], b["db"][i])


@pytest.mark.parametrize("C", [4096 + 37, 256 * 272 + 37], ids=["thin-tiles", "mixed-tiles"])
def test_recomputed_logits_are_the_forward_logits_bit_for_bit(H, C):
    """The backward call recomputes the logits; they must be the forward call's, bit for bit, whichever
    kind of tile computed them.  Two chains of exact comparisons, all through the C ABI:

    fp32, exact: a shard's row_max from the forward call (thin tiles, or full and thin mixed) equals the
    best logit the arg-max call reports (full tiles only), and with every label set to that arg-max class
    the label logit equals both.

    dz, exact at bf16: with B <= D / 2, features [D/2 + i] = 1 in row i only, dW[c, D/2 + i] is
    dz[i, c] itself (one non-zero term, a bf16 number times 1).  With g = 1 it must equal, off the label,
    the prediction exp(z - lse) that the predictions call (full tiles only) writes for the same lse.  The
    other D / 2 features are random, so the logits are sums whose rounding depends on the order of the
    contraction: one differing fp32 bit flips a bf16 rounding once in ~2^16 elements, and there are 1e6
    (thin) or 1.8e7 (mixed) of them."""
    import torch
    from paper_2011_09208_amd import binding as ws
    B, D = 256, 1024
    p = inputs.make_inputs("recompute", B, D, C, x_sigma=1.0, w_sigma=0.05, bias_sigma=0.5, seed=C)
    X = inputs.bf16_bits_to_f32(p.X_bits).copy()
    X[:, D // 2:] = 0.0
    X[np.arange(B), D // 2 + np.arange(B)] = 1.0
    p.X_bits = inputs.f32_to_bf16_bits(X)
    H.say(f"[parity] recompute == forward: B={B} D={D} C={C}")
    dev = torch.device("cuda")
    Xd, Wd = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).to(dev)
    work = torch.empty(max(ws.fwd_workspace_bytes(B, D, C), ws.bwd_workspace_bytes(B, D, C)), dtype=torch.uint8,
                       device=dev)
    tv = torch.empty(B, device=dev)
    tc = torch.empty(B, device=dev, dtype=torch.int32)
    ws.split_fc_top1(Xd, Wd, bias, 0, tv, tc, work)
    m, s, t = (torch.empty((1, B), device=dev) for _ in range(3))
    lse, loss = torch.empty(B, device=dev), torch.empty(B, device=dev)
    ws.split_fc_fwd(Xd, Wd, bias, tc, 0, m[0], s[0], t[0], work)          # labels = the arg-max classes
    ws.combine_partials(m, s, t, lse, loss, None)
    torch.cuda.synchronize()
    assert torch.equal(m[0].view(torch.int32), tv.view(torch.int32))
    assert torch.equal(t[0].view(torch.int32), tv.view(torch.int32))
    P = torch.empty((B, (C + 7) // 8 * 8), device=dev, dtype=torch.bfloat16)
    ws.split_fc_predict(Xd, Wd, bias, lse, P[:, :C])
    dX = torch.empty((B, D), device=dev)
    dW = torch.empty((C, D), device=dev, dtype=torch.bfloat16)
    ws.split_fc_bwd(Xd, Wd, bias, lse, tc, 0, 1.0, dX, False, dW, None, work)
    torch.cuda.synchronize()
    dz = dW[:, D // 2: D // 2 + B].t().contiguous().view(torch.int16)      # [B, C]
    pr = P[:, :C].contiguous().view(torch.int16)
    off_label = torch.ones((B, C), dtype=torch.bool, device=dev)
    off_label[torch.arange(B, device=dev), tc.long()] = False
    differing = int(((dz != pr) & off_label).sum())
    H.say(f"[parity] recompute == forward: {differing} of {B * C - B} off-label dz elements differ from the predictions")
    assert differing == 0
    # at the label dz = p - 1 <= 0
    at_label = dW[tc.long(), D // 2 + torch.arange(B, device=dev)].float()
    assert bool((at_label <= 0).all()) and bool((at_label >= -1).all())
    H.record(f"recompute == forward C={C}", f"B={B} D={D} C={C}", {"off_label_dz_elements_differing": differing})


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "headline"])
def test_full_size_workloads(H, name):
    """The paper-shaped workloads at full size, every output compared element by element."""
    p = inputs.make_config(name)
    _full_parity(H, p, p.shards, tag=name, gate="stated")


def _wide_layer_parity(H, name, g, rows_per_chunk):
    """A layer too wide for the [B, C] fp64 logits to sit in host memory at once: every shard's forward call,
    the combine, every shard's backward call (dX accumulated over the shards) on the GPU, against the oracle's
    unsharded definition evaluated in row blocks.  Compared: every shard's statistics are merged by the
    library, so lse and loss of every row (stated gates); the summed dX and every shard's db element by
    element; dW of the first shard element by element against the oracle's shard gradients for the oracle's
    own log-sum-exp (the other shards' dW stay on the device: gigabytes on the host as fp64); the first
    shard's forward statistics against the oracle's partials."""
    from oracle import oracle
    p = inputs.make_config(name)
    S = len(p.shards)
    shape = f"B={p.B} D={p.D} C={p.C} shards={S} g={g:.3g}"
    H.say(f"[parity] {name} whole layer: {shape}")
    X = inputs.bf16_bits_to_f64(p.X_bits)
    W = inputs.bf16_bits_to_f64(p.W_bits)
    y = p.labels.astype(np.int64)
    got = H.run_step(p.X_bits, p.W_bits, None, p.labels, p.shards, g=g, keep_dW=[0])
    H.say(f"[parity] {name} whole layer: GPU step done, oracle in blocks of {rows_per_chunk} rows")
    ref = oracle.unsharded_chunked(X, W, None, y, g, rows_per_chunk=rows_per_chunk, want_dW=False)
    rep = {}
    rep["lse_abs"] = float(np.max(np.abs(got["lse"] - ref["lse"])))
    rep["loss_rel"] = float(np.max(np.abs(got["loss"] - ref["loss"]) / np.abs(ref["loss"])))
    assert rep["lse_abs"] <= H.LSE_ABS, rep
    assert rep["loss_rel"] <= H.LOSS_REL, rep
    owners = np.zeros(p.B, dtype=int)
    for i, (off, c) in enumerate(p.shards):
        inside = (y >= off) & (y < off + c)
        owners += inside
        assert np.all(got["t"][i][~inside] == 0.0)
    assert np.array_equal(owners, np.ones(p.B, dtype=int))
    off, c = p.shards[0]
    m0, s0, t0 = oracle.partials(X, W[off:off + c], None, y, off)
    rep["row_max_abs"] = float(np.max(np.abs(got["m"][0] - m0)))
    rep["sumexp_rel"] = float(np.max(np.abs(got["s"][0] - s0) / s0))
    rep["label_logit_abs"] = float(np.max(np.abs(got["t"][0] - t0)))
    assert rep["row_max_abs"] <= H.LSE_ABS and rep["sumexp_rel"] <= 1e-3 and rep["label_logit_abs"] <= H.LSE_ABS, rep
    rep["dX"] = H.max_rel_to_max(got["dX"], ref["dX"])
    rep["db"] = H.max_rel_to_max(np.concatenate(got["db"]), ref["db"])
    g0 = oracle.shard_grads(X, W[off:off + c], None, ref["lse"], y, off, g)
    rep["dW"] = H.max_rel_to_max(got["dW"][0], g0["dW"])
    H.say(f"[parity] {name} whole layer: " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()))
    H.record(f"{name} whole layer", shape + " gate=stated", rep)
    for k in ("dX", "dW", "db"):
        assert rep[k] <= H.GRAD_REL_TO_MAX, (k, rep)


def test_large_vocab_head_all_shards(H):
    """cfg5 at full size: B = 8192 token rows, D = 1024, all 8 shards of the 400 000-class output run one
    after another and combined, Zipf labels (most of them in the first shard), mean-loss gradient scale."""
    _wide_layer_parity(H, "cfg5", 1.0 / 8192, rows_per_chunk=512)


def test_million_class_layer_all_shards(H):
    """The paper's second workload (Section 5.1.2): a 1M-class layer cut 8 ways, B = 1024, D = 2048; all 8
    shards (C_shard = 125 000) run one after another and combined."""
    _wide_layer_parity(H, "million", 1.0, rows_per_chunk=256)


def test_widest_shard_the_32bit_offsets_allow(H):
    """The kernels address an operand with 32-bit byte offsets, so a shard's weight matrix (plus 256 rows of
    slack) must stay below 4 GiB; this runs the widest legal shard at D = 2048 — 1 048 000 classes, 4.29 GB of
    weights, offsets up to 2^32 - 1.3e6 — through forward, combine and backward.  The oracle evaluates the layer
    in blocks of 65 536 classes (its per-shard functions, combined by its own merge): lse and loss of every row,
    the summed dX, db of every class and dW of the last block (the rows with the largest offsets) are compared
    element by element."""
    from oracle import oracle
    B, D, C = 256, 2048, 1_048_000
    p = inputs.make_inputs("widest", B, D, C, x_relu=True, w_sigma=0.01, seed=11)
    H.say(f"[parity] widest shard: B={B} D={D} C_shard={C} ({C * D * 2 / 2**30:.2f} GiB of weights)")
    g = 1.0 / B
    got = H.run_step(p.X_bits, p.W_bits, None, p.labels, [(0, C)], g=g, keep_dW=[])
    X = inputs.bf16_bits_to_f64(p.X_bits)
    y = p.labels.astype(np.int64)
    blocks = [(o, min(65_536, C - o)) for o in range(0, C, 65_536)]
    stats = [oracle.partials(X, inputs.bf16_bits_to_f64(p.W_bits[o:o + c]), None, y, o) for o, c in blocks]
    lse, loss = oracle.combine(*zip(*stats))
    rep = {"lse_abs": float(np.max(np.abs(got["lse"] - lse))),
           "loss_rel": float(np.max(np.abs(got["loss"] - loss) / np.abs(loss)))}
    assert rep["lse_abs"] <= H.LSE_ABS and rep["loss_rel"] <= H.LOSS_REL, rep
    dX = np.zeros((B, D))
    db = np.empty(C)
    for o, c in blocks:
        gr = oracle.shard_grads(X, inputs.bf16_bits_to_f64(p.W_bits[o:o + c]), None, lse, y, o, g)
        dX += gr["dX_partial"]
        db[o:o + c] = gr["db"]
    rep["dX"] = H.max_rel_to_max(got["dX"], dX)
    rep["db"] = H.max_rel_to_max(got["db"][0], db)
    # dW of the last block, read back from the device separately (the whole dW is 4.3 GB)
    import torch
    from paper_2011_09208_amd import binding as ws
    o, c = blocks[-1]
    Xd, Wd = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    yd = torch.from_numpy(p.labels).cuda()
    lsed = torch.from_numpy(lse.astype(np.float32)).cuda()
    dXd = torch.empty((B, D), device="cuda")
    dWd = torch.empty((C, D), device="cuda", dtype=torch.bfloat16)
    work = torch.empty(ws.bwd_workspace_bytes(B, D, C), dtype=torch.uint8, device="cuda")
    ws.split_fc_bwd(Xd, Wd, None, lsed, yd, 0, g, dXd, False, dWd, None, work)
    torch.cuda.synchronize()
    rep["dW_last_block"] = H.max_rel_to_max(H.bf16_to_f64(dWd[o:o + c]), gr["dW"])
    rep["dW_first_block"] = H.max_rel_to_max(
        H.bf16_to_f64(dWd[:65_536]),
        oracle.shard_grads(X, inputs.bf16_bits_to_f64(p.W_bits[:65_536]), None, lse, y, 0, g)["dW"])
    H.say("[parity] widest shard: " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()))
    H.record("widest shard (32-bit offset limit)", f"B={B} D={D} C={C} g={g:.3g} gate=stated", rep)
    for k in ("dX", "db", "dW_last_block", "dW_first_block"):
        assert rep[k] <= H.GRAD_REL_TO_MAX, (k, rep)


def test_padded_pitches_stream_and_accumulate(H):
    """Row pitches larger than the row length for every matrix argument, a side stream, loss_mean, and
    accumulate_dx on top of a pre-filled dX: the library must honour pitches, touch nothing in the padding,
    enqueue on the stream it is given, and add to (not overwrite) dX when asked."""
    import torch
    from oracle import oracle
    from paper_2011_09208_amd import binding as ws
    B, D, C = 200, 128, 700
    p = inputs.make_inputs("pitch", B, D, C, w_sigma=0.3, bias_sigma=0.7, seed=21)
    H.say(f"[parity] padded pitches on a side stream: B={B} D={D} C={C}")
    dev = torch.device("cuda")
    PX, PW, PDX, PDW = D + 64, D + 8, D + 12, D + 24
    Xp = torch.full((B, PX), float("nan"), device=dev, dtype=torch.bfloat16)
    Xp[:, :D] = H.dev_bf16(p.X_bits)
    Wp = torch.full((C, PW), float("nan"), device=dev, dtype=torch.bfloat16)
    Wp[:, :D] = H.dev_bf16(p.W_bits)
    X, W = Xp[:, :D], Wp[:, :D]
    bias = torch.from_numpy(p.bias).to(dev)
    y = torch.from_numpy(p.labels).to(dev)
    m, s, t = (torch.empty((1, B), device=dev) for _ in range(3))
    lse, loss, mean = torch.empty(B, device=dev), torch.empty(B, device=dev), torch.empty(1, device=dev)
    dXp = torch.full((B, PDX), 7.0, device=dev)
    dWp = torch.full((C, PDW), 3.0, device=dev, dtype=torch.bfloat16)
    db = torch.empty(C, device=dev)
    work = torch.empty(max(ws.fwd_workspace_bytes(B, D, C), ws.bwd_workspace_bytes(B, D, C)), dtype=torch.uint8,
                       device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ws.split_fc_fwd(X, W, bias, y, 0, m[0], s[0], t[0], work)
        ws.combine_partials(m, s, t, lse, loss, mean)
        ws.split_fc_bwd(X, W, bias, lse, y, 0, 0.5, dXp[:, :D], True, dWp[:, :D], db, work)
    side.synchronize()
    ref = oracle.unsharded(inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits),
                           p.bias.astype(np.float64), p.labels, 0.5)
    assert np.max(np.abs(lse.cpu().numpy() - ref["lse"])) <= H.LSE_ABS * max(1.0, np.abs(ref["lse"]).max())
    assert abs(float(mean.cpu()[0]) - ref["loss_mean"]) <= 1e-3 * ref["loss_mean"]
    dX = dXp.cpu().numpy()
    assert np.all(dX[:, D:] == 7.0)                                   # padding untouched
    assert H.max_rel_to_max(dX[:, :D] - 7.0, ref["dX"]) <= H.GRAD_REL_TO_MAX + 1e-5    # accumulated on top of 7
    dW = dWp.float().cpu().numpy()
    assert np.all(dW[:, D:] == 3.0)
    assert H.max_rel_to_max(dW[:, :D].astype(np.float64), ref["dW"]) <= H.GRAD_REL_TO_MAX
    assert H.max_rel_to_max(db.cpu().numpy(), ref["db"]) <= H.GRAD_REL_TO_MAX
    assert torch.isnan(Xp[:, D:]).all() and torch.isnan(Wp[:, D:]).all()      # inputs never modified


def test_graph_capture_replays_match_eager(H):
    """The three calls allocate nothing, never synchronise and clear no memory with memset nodes, so a
    whole step can be captured into a HIP graph.  Every replay (with the program's own eager work and
    synchronisations between the replays) must reproduce the eager results bit for bit."""
    import torch
    from paper_2011_09208_amd import binding as ws
    p = inputs.make_inputs("graph", 300, 256, 3000, w_sigma=0.2, bias_sigma=0.5, seed=33)
    H.say(f"[parity] graph capture: B={p.B} D={p.D} C={p.C}, two shards")
    dev = torch.device("cuda")
    shards = [(0, 1100), (1100, 1900)]
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).to(dev)
    y = torch.from_numpy(p.labels).to(dev)
    B, D = p.B, p.D
    m, s, t = (torch.empty((2, B), device=dev) for _ in range(3))
    lse, loss, mean = torch.empty(B, device=dev), torch.empty(B, device=dev), torch.empty(1, device=dev)
    dX = torch.empty((B, D), device=dev)
    dW = torch.empty((p.C, D), device=dev, dtype=torch.bfloat16)
    db = torch.empty(p.C, device=dev)
    work = torch.empty(max(max(ws.fwd_workspace_bytes(B, D, c), ws.bwd_workspace_bytes(B, D, c)) for _, c in shards),
                       dtype=torch.uint8, device=dev)
    outs = (m, s, t, lse, loss, mean, dX, dW, db)

    def step():
        for i, (off, c) in enumerate(shards):
            ws.split_fc_fwd(X, W[off:off + c], bias[off:off + c], y, off, m[i], s[i], t[i], work)
        ws.combine_partials(m, s, t, lse, loss, mean)
        for i, (off, c) in enumerate(shards):
            ws.split_fc_bwd(X, W[off:off + c], bias[off:off + c], lse, y, off, 0.25, dX, i > 0, dW[off:off + c],
                            db[off:off + c], work)

    step()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan")) if o.dtype != torch.bfloat16 else o.fill_(1.0)
        work.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o.view(torch.int16) if o.dtype == torch.bfloat16 else o.view(torch.int32),
                               e.view(torch.int16) if e.dtype == torch.bfloat16 else e.view(torch.int32)), rep
    ref = H.oracle_step(p.X_bits, p.W_bits, p.bias, p.labels, shards, g=0.25)
    assert np.max(np.abs(lse.cpu().numpy() - ref["lse"])) <= H.LSE_ABS * max(1.0, np.abs(ref["lse"]).max())
    assert H.max_rel_to_max(dX.cpu().numpy(), ref["dX"]) <= H.GRAD_REL_TO_MAX


def _predict_parity(H, p, shards, pad=0, tag=""):
    """Predictions of every shard against the oracle's, given the oracle's combined log-sum-exp rounded
    to fp32 (an input).  Relative gate: bf16 rounding of P (2^-9) plus the effect of the logits' own
    fp32 rounding on exp (the lse gate, scaled like it), plus a floor for values that underflow bf16."""
    import torch
    from oracle import oracle
    from paper_2011_09208_amd import binding as ws
    X64, W64 = inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits)
    b64 = None if p.bias is None else p.bias.astype(np.float64)
    Z = oracle.logits(X64, W64, b64)
    lse32 = oracle.logsumexp_rows(Z).astype(np.float32)
    zscale = max(1.0, float(np.max(np.abs(Z))))
    del Z
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = None if p.bias is None else torch.from_numpy(p.bias).cuda()
    lse = torch.from_numpy(lse32).cuda()
    worst = 0.0
    row_sum = np.zeros(p.B)
    for off, c in shards:
        ldp = (c + 7) // 8 * 8 + pad
        Pbuf = torch.full((p.B, ldp), 3.0, dtype=torch.bfloat16, device="cuda")
        P = Pbuf[:, :c]
        ws.split_fc_predict(X, W[off:off + c], None if bias is None else bias[off:off + c], lse, P)
        torch.cuda.synchronize()
        got = H.bf16_to_f64(Pbuf)
        assert np.all(got[:, c:] == 3.0), f"{tag}: columns beyond the shard were written"
        ref = oracle.predictions(X64, W64[off:off + c], None if b64 is None else b64[off:off + c],
                                 lse32.astype(np.float64))
        err = np.abs(got[:, :c] - ref)
        tol = (2.0 ** -8 + 2 * H.LSE_ABS * zscale) * ref + 1e-38
        assert np.all(err <= tol), (tag, off, c, float(np.max(err / (ref + 1e-300))))
        worst = max(worst, float(np.max(err / (ref + 1e-30))))
        row_sum += got[:, :c].sum(axis=1)
    assert np.max(np.abs(row_sum - 1.0)) <= 2.0 ** -8 + 2 * H.LSE_ABS * zscale, tag
    H.say(f"[parity] {tag}: predictions max rel err {worst:.2e}, max |row sum - 1| {np.max(np.abs(row_sum - 1.0)):.2e}")


def test_predictions_small_and_ragged(H):
    p = inputs.make_config("cfg1")
    H.say("[parity] predictions cfg1")
    _predict_parity(H, p, p.shards, tag="predict cfg1")
    for B, D, C, shards, seed in [(300, 128, 777, [(0, 5), (5, 515), (520, 257)], 41),
                                  (257, 64, 1031, [(0, 1031)], 42),
                                  (1, 64, 9, [(0, 1), (1, 8)], 43)]:
        q = inputs.make_inputs("predict", B, D, C, w_sigma=0.4, bias_sigma=1.0, seed=seed)
        H.say(f"[parity] predictions ragged: B={B} D={D} C={C} shards={shards}")
        _predict_parity(H, q, shards, pad=8, tag=f"predict {B}x{D}x{C}")


def test_predictions_full_size_uneven_shards(H):
    """cfg4 at full size: B = 1024, D = 2048, C = 100 000 as the uneven shards (37 500, 12 500, 37 500, 12 500),
    every element of every shard against the oracle."""
    p = inputs.make_config("cfg4")
    H.say(f"[parity] predictions cfg4: B={p.B} D={p.D} C={p.C} shards={p.shards}")
    _predict_parity(H, p, p.shards, tag="predict cfg4")


def _fused_sgd_parity(H, p, shards, lr, g, tag):
    """ws_split_fc_bwd_sgd against the oracle's update: the new weights within bf16 rounding of the result
    plus the gradient gate times lr, the new bias likewise in fp32, and dX bit for bit what the plain
    backward call gives (it must use the weights from before the update)."""
    import torch
    from oracle import oracle
    from paper_2011_09208_amd import binding as ws
    H.say(f"[parity] fused SGD {tag}: B={p.B} D={p.D} C={p.C} shards={shards} lr={lr} g={g:.3g}")
    dev = torch.device("cuda")
    X = H.dev_bf16(p.X_bits)
    y = torch.from_numpy(p.labels).to(dev)
    B, D, S = p.B, p.D, len(shards)
    m, s, t = (torch.empty((S, B), device=dev) for _ in range(3))
    lse, loss = torch.empty(B, device=dev), torch.empty(B, device=dev)
    work = torch.empty(max(max(ws.fwd_workspace_bytes(B, D, c), ws.bwd_workspace_bytes(B, D, c)) for _, c in shards),
                       dtype=torch.uint8, device=dev)
    PW = D + 8                                     # padded pitch: the padding must stay untouched
    Wp = torch.full((p.C, PW), 5.0, device=dev, dtype=torch.bfloat16)
    Wp[:, :D] = H.dev_bf16(p.W_bits)
    W = Wp[:, :D]
    bias = None if p.bias is None else torch.from_numpy(p.bias).to(dev)
    bsl = lambda off, c: None if bias is None else bias[off:off + c]
    for i, (off, c) in enumerate(shards):
        ws.split_fc_fwd(X, W[off:off + c], bsl(off, c), y, off, m[i], s[i], t[i], work)
    ws.combine_partials(m, s, t, lse, loss, None)
    # plain backward first (keeps W), then the fused one
    dX_ref = torch.empty((B, D), device=dev)
    dW = torch.empty((p.C, D), device=dev, dtype=torch.bfloat16)
    db = torch.empty(p.C, device=dev)
    for i, (off, c) in enumerate(shards):
        ws.split_fc_bwd(X, W[off:off + c], bsl(off, c), lse, y, off, g, dX_ref, i > 0, dW[off:off + c],
                        db[off:off + c], work)
    dX = torch.full((B, D), float("nan"), device=dev)
    for i, (off, c) in enumerate(shards):
        ws.split_fc_bwd_sgd(X, W[off:off + c], bsl(off, c), lse, y, off, g, lr, dX, i > 0, work)
    torch.cuda.synchronize()
    assert torch.equal(dX.view(torch.int32), dX_ref.view(torch.int32))
    W64, X64 = inputs.bf16_bits_to_f64(p.W_bits), inputs.bf16_bits_to_f64(p.X_bits)
    b64 = None if p.bias is None else p.bias.astype(np.float64)
    ref = oracle.unsharded(X64, W64, b64, p.labels.astype(np.int64), g)
    Wn, bn = oracle.sgd_update(W64, b64, ref["dW"], ref["db"], lr)
    got_W = H.bf16_to_f64(Wp)
    assert np.all(got_W[:, D:] == 5.0)
    tol_W = 2.0 ** -8 * np.abs(Wn) + abs(lr) * H.GRAD_REL_TO_MAX * np.max(np.abs(ref["dW"]))
    err_W = np.abs(got_W[:, :D] - Wn)
    assert np.all(err_W <= tol_W), float(np.max(err_W))
    assert np.abs(got_W[:, :D] - W64).max() > 0                      # the update did something
    if bias is not None:
        got_b = bias.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got_b - bn) <= 1e-6 * np.abs(bn) + abs(lr) * H.GRAD_REL_TO_MAX * np.max(np.abs(ref["db"])))
    # the fused call equals "plain backward, then W - lr * (its bf16 dW), rounded to bf16" up to the last
    # bit of a few entries (the kernel uses one fused multiply-add, numpy a multiply and an add)
    two_step = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(p.W_bits)
                                       + np.float32(-lr) * H.bf16_to_f64(dW).astype(np.float32))
    agree = (got_W[:, :D] == inputs.bf16_bits_to_f64(two_step)).mean()
    assert agree > 0.999, agree
    H.record(f"fused SGD {tag}", f"B={B} D={D} C={p.C} shards={S} lr={lr} g={g:.3g}",
             {"W_new_max_abs_err": float(np.max(err_W)), "W_new_max_err_over_tol": float(np.max(err_W / tol_W)),
              "bitwise_agreement_with_two_step": float(agree)})


@pytest.mark.parametrize("B,D,widths,seed", [
    (300, 256, [700, 800], 61),                 # thin tiles only
    (300, 64, [256 * 70 + 5], 62),              # 142 full tiles, ragged batch and class edge
    (513, 64, [256 * 90 + 17], 63),             # 256 full + 68 thin tiles
    (300, 1024, [256 * 70 + 5], 64),            # dW kernel: 284 tiles, more than one round
    (3100, 320, [600], 65),                     # dW kernel: long contraction, thin tiles
], ids=["thin", "full-tiles", "mixed-tiles", "mixed-dw-tiles", "long-k-dw-thin"])
def test_backward_with_fused_sgd_update(H, B, D, widths, seed):
    C = sum(widths)
    p = inputs.make_inputs("sgd", B, D, C, w_sigma=0.3, bias_sigma=0.5, seed=seed)
    shards, o = [], 0
    for w in widths:
        shards.append((o, w))
        o += w
    _fused_sgd_parity(H, p, shards, lr=0.05, g=1.0 / B, tag=f"{B}x{D}x{C}")


def test_backward_with_fused_sgd_update_headline_size(H):
    """The fused update at the headline shape (B = 1024, D = 2048, C = 100 000, no bias), every weight
    against the oracle's.  The gradients of the mean loss are ~1e-5 there, so the learning rate is chosen
    large enough for the update to move bf16 weights of magnitude 0.01."""
    p = inputs.make_config("headline")
    _fused_sgd_parity(H, p, p.shards, lr=50.0, g=1.0 / p.B, tag="headline")


def _top1_run(H, X_bits, W_bits, bias, shards):
    import torch
    from paper_2011_09208_amd import binding as ws
    X, W = H.dev_bf16(X_bits), H.dev_bf16(W_bits)
    B, D = X.shape
    b = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    S = len(shards)
    tv = torch.full((S, B), float("nan"), device="cuda")
    tc = torch.full((S, B), -7, device="cuda", dtype=torch.int32)
    work = torch.empty(max(ws.fwd_workspace_bytes(B, D, c) for _, c in shards), dtype=torch.uint8, device="cuda")
    work.fill_(0xFF)
    for i, (off, c) in enumerate(shards):
        ws.split_fc_top1(X, W[off:off + c], None if b is None else b[off:off + c], off, tv[i], tc[i], work)
    bv = torch.full((B,), float("nan"), device="cuda")
    bc = torch.full((B,), -7, device="cuda", dtype=torch.int32)
    ws.combine_top1(tv, tc, bv, bc)
    torch.cuda.synchronize()
    return tv.cpu().numpy(), tc.cpu().numpy(), bv.cpu().numpy(), bc.cpu().numpy()


def test_top1_exact_cases(H):
    """Integer-valued logits are exact in fp32, so the arg-max and the tie rule can be checked bit for bit:
    W = 0 and b_c = c gives the last class of every shard; a constant bias ties all classes and the lowest id
    must win, inside a shard and across shards."""
    B, D, C = 70, 64, 1000
    shards = [(0, 300), (300, 1), (301, 699)]
    Xb = inputs.make_inputs("top1", B, D, C, seed=71).X_bits
    Wz = np.zeros((C, D), dtype=np.uint16)
    H.say("[parity] top-1: exact integer logits and ties")
    tv, tc, bv, bc = _top1_run(H, Xb, Wz, np.arange(C, dtype=np.float32), shards)
    for i, (off, c) in enumerate(shards):
        assert np.all(tc[i] == off + c - 1) and np.all(tv[i] == float(off + c - 1))
    assert np.all(bc == C - 1) and np.all(bv == float(C - 1))
    tv, tc, bv, bc = _top1_run(H, Xb, Wz, np.full(C, 3.0, dtype=np.float32), shards)
    for i, (off, c) in enumerate(shards):
        assert np.all(tc[i] == off) and np.all(tv[i] == 3.0)
    assert np.all(bc == 0)
    # descending bias: the first class of every shard, and class 0 overall
    tv, tc, bv, bc = _top1_run(H, Xb, Wz, -np.arange(C, dtype=np.float32), shards)
    assert np.all(tc == np.array([o for o, _ in shards])[:, None]) and np.all(bc == 0)


def _top1_parity(H, p, shards, tag):
    from oracle import oracle
    H.say(f"[parity] {tag}: top-1 B={p.B} D={p.D} C={p.C} shards={shards if len(shards) < 6 else len(shards)}")
    tv, tc, bv, bc = _top1_run(H, p.X_bits, p.W_bits, p.bias, shards)
    X64, W64 = inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits)
    b64 = None if p.bias is None else p.bias.astype(np.float64)
    Z = oracle.logits(X64, W64, b64)
    tol = H.LSE_ABS * max(1.0, float(np.max(np.abs(Z))))
    rows = np.arange(p.B)
    refs = []
    for i, (off, c) in enumerate(shards):
        rv, rc = oracle.top1(X64, W64[off:off + c], None if b64 is None else b64[off:off + c], off)
        refs.append((rv, rc))
        assert np.all((tc[i] >= off) & (tc[i] < off + c))
        assert np.max(np.abs(tv[i] - rv)) <= tol                       # the best logit itself
        assert np.all(Z[rows, tc[i]] >= rv - 2 * tol)                  # the chosen class is a maximum up to rounding
        part = np.partition(Z[:, off:off + c], -2, axis=1) if c > 1 else None
        clear = np.ones(p.B, dtype=bool) if c == 1 else (part[:, -1] - part[:, -2] > 2 * tol)
        assert np.array_equal(tc[i][clear], rc[clear])                 # exact wherever the decision is not a near-tie
    rbv, rbc = oracle.combine_top1([r[0] for r in refs], [r[1] for r in refs])
    part = np.partition(Z, -2, axis=1)
    clear = part[:, -1] - part[:, -2] > 2 * tol
    assert np.max(np.abs(bv - rbv)) <= tol and np.array_equal(bc[clear], rbc[clear])
    assert np.all(Z[rows, bc] >= rbv - 2 * tol)
    # the merge itself is integer work on the candidates it was given: bit-exact against the oracle's merge
    mv, mc = oracle.combine_top1(list(tv.astype(np.float64)), list(tc.astype(np.int64)))
    assert np.array_equal(mc, bc) and np.array_equal(mv.astype(np.float32), bv)
    H.say(f"[parity] {tag}: top-1 clear rows {int(clear.sum())} of {p.B}, all agree")


def test_top1_ragged_and_full_size(H):
    q = inputs.make_inputs("top1", 300, 128, 1031, w_sigma=0.4, bias_sigma=1.0, seed=72)
    _top1_parity(H, q, [(0, 5), (5, 515), (520, 511)], "ragged")
    p = inputs.make_config("cfg4")
    _top1_parity(H, p, p.shards, "cfg4")


def test_ceiling_probes_compute_what_they_time(H):
    """The diagnostic GEMM (the library's main loop alone) against the oracle's logits, which is the same
    product X . W^T, within bf16 rounding of the output; the MFMA-only loop leaves an exactly known checksum
    for all-ones operands (every MFMA adds 32 to each of a wave's accumulator elements)."""
    import torch
    from oracle import oracle
    from paper_2011_09208_amd import binding as ws
    M, N, K = 512, 768, 320
    p = inputs.make_inputs("probe", M, K, N, x_sigma=1.0, w_sigma=0.5, seed=90)      # X [M, K], W [N, K]
    H.say(f"[parity] probe GEMM {M} x {N} x {K}")
    A, Bm = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    Cm = torch.full((N, M), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws.probe_gemm(A, Bm, Cm)
    torch.cuda.synchronize()
    ref = oracle.logits(inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits)).T       # [N, M]
    got = H.bf16_to_f64(Cm)
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4)
    rounds, wgs = 3, 5
    frag = torch.ones(16 * 512 * 8, device="cuda", dtype=torch.bfloat16)
    sink = torch.full((wgs * 512,), float("nan"), device="cuda")
    ws.probe_mfma_loop(frag, rounds, wgs, sink)
    torch.cuda.synchronize()
    # per lane: 16 accumulators x 4 elements, each rounds x 8 MFMAs x 32
    assert torch.equal(sink, torch.full_like(sink, 16 * 4 * rounds * 8 * 32.0))


def test_traced_dw_kernel_writes_the_same_gradients(H):
    """The instrumented copy of the dW kernel (per-tile clock stamps for the benchmark's trace) must leave
    every output bit for bit as the plain kernel does, stamp every tile once with clocks that never run
    backwards, and refuse a trace buffer that is too small before launching anything."""
    import torch
    from paper_2011_09208_amd import binding as ws
    B, D, C = 300, 512, 17925            # 2 feature tiles x 71 class tiles, ragged in rows and classes
    p = inputs.make_inputs("trace", B, D, C, x_sigma=1.0, w_sigma=0.2, bias_sigma=0.5, seed=17)
    H.say(f"[parity] traced dW kernel: B={B} D={D} C={C}")
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).cuda()
    y = torch.from_numpy(np.ascontiguousarray(p.labels, dtype=np.int32)).cuda()
    work = torch.empty(max(ws.fwd_workspace_bytes(B, D, C), ws.bwd_workspace_bytes(B, D, C)), dtype=torch.uint8,
                       device="cuda")
    m, s, t, lse, loss = (torch.empty(B, device="cuda") for _ in range(5))
    ws.split_fc_fwd(X, W, bias, y, 0, m, s, t, work)
    ws.combine_partials(m.view(1, B), s.view(1, B), t.view(1, B), lse, loss, None)

    def bwd():
        dX = torch.full((B, D), float("nan"), device="cuda")
        dW = torch.full((C, D), float("nan"), device="cuda", dtype=torch.bfloat16)
        db = torch.full((C,), float("nan"), device="cuda")
        ws.split_fc_bwd(X, W, bias, lse, y, 0, 1.0 / B, dX, False, dW, db, work)
        torch.cuda.synchronize()
        return dX, dW, db

    plain = bwd()
    tiles = (D // 256) * (-(-C // 256))
    trace = torch.zeros((tiles, 8), dtype=torch.int64, device="cuda")
    try:
        ws.profile_trace_dw(trace[:tiles - 1].contiguous())
        with pytest.raises(ws.WhaleSplitError) as err:
            bwd()
        assert err.value.status == 5                      # WS_ERR_WORKSPACE
        ws.profile_trace_dw(trace)
        traced = bwd()
    finally:
        ws.profile_trace_dw(None)
    again = bwd()
    for a, b, c in zip(plain, traced, again):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32),
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32))
        assert torch.equal(b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32),
                           c.view(torch.int16) if c.dtype == torch.bfloat16 else c.view(torch.int32))
    tr = trace.cpu().numpy()
    assert np.all(tr[:, 0] > 0) and np.all(np.diff(tr[:, :6], axis=1) >= 0)
    assert len(np.unique(tr[:, 6])) == tiles              # one workgroup per tile
