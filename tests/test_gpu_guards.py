"""GPU: every entry point writes its outputs and nothing else.

Each output (and the workspace, sized exactly as the size query says) sits inside a larger allocation
whose surroundings, and the padding columns of pitched matrices, hold a byte pattern.  After the calls
the pattern must be intact everywhere outside the payload, and the payload must equal, bit for bit,
what the same calls produce into plain buffers.  The shapes cover launches of thin tiles only, of
full tiles only and of both, with ragged row and class counts (where a tile hangs over the edge of
its output)."""
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


def Guarded(*a, **kw):
    from tests.gpu_harness import Guarded as G
    return G(*a, **kw)


def _bits(t):
    import torch
    return t.contiguous().view({1: torch.uint8, 2: torch.int16, 4: torch.int32}[t.element_size()])


SHAPES = [
    ("thin tiles only", 300, 64, 1000),
    ("full tiles only", 300, 64, 17925),
    ("full and thin tiles", 513, 64, 23057),
    ("five batch tiles", 1100, 128, 14000),
    ("dW in full and thin tiles", 300, 1024, 17925),
    ("dW in thin tiles, long contraction", 3100, 320, 600),
]


@pytest.mark.parametrize("tag,B,D,C", SHAPES, ids=[s[0].replace(" ", "-") for s in SHAPES])
def test_step_writes_only_its_outputs(H, tag, B, D, C):
    import torch
    from paper_2011_09208_amd import binding as ws
    p = inputs.make_inputs("guards", B, D, C, x_sigma=1.0, w_sigma=0.2, bias_sigma=0.5, seed=B + C)
    H.say(f"[guards] {tag}: B={B} D={D} C={C}")
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).cuda()
    y = torch.from_numpy(np.ascontiguousarray(p.labels, dtype=np.int32)).cuda()
    off = 0
    nws = max(ws.fwd_workspace_bytes(B, D, C), ws.bwd_workspace_bytes(B, D, C))

    def outputs(guarded):
        if guarded:
            g = dict(m=Guarded(1, B, torch.float32), s=Guarded(1, B, torch.float32), t=Guarded(1, B, torch.float32),
                     lse=Guarded(1, B, torch.float32), loss=Guarded(1, B, torch.float32),
                     mean=Guarded(1, 1, torch.float32), dX=Guarded(B, D, torch.float32, pad_cols=8),
                     dW=Guarded(C, D, torch.bfloat16, pad_cols=8), db=Guarded(1, C, torch.float32),
                     P=Guarded(B, C, torch.bfloat16, pad_cols=(-C) % 8 + 8),
                     top=Guarded(1, B, torch.float32), cls=Guarded(1, B, torch.int32),
                     work=Guarded(1, nws, torch.uint8))
            return g, {k: (v.t if v.rows > 1 else v.vec()) for k, v in g.items()}
        t = dict(m=torch.empty(B, device="cuda"), s=torch.empty(B, device="cuda"), t=torch.empty(B, device="cuda"),
                 lse=torch.empty(B, device="cuda"), loss=torch.empty(B, device="cuda"),
                 mean=torch.empty(1, device="cuda"), dX=torch.empty((B, D), device="cuda"),
                 dW=torch.empty((C, D), device="cuda", dtype=torch.bfloat16), db=torch.empty(C, device="cuda"),
                 P=torch.empty((B, C + (-C) % 8), device="cuda", dtype=torch.bfloat16)[:, :C],
                 top=torch.empty(B, device="cuda"), cls=torch.empty(B, device="cuda", dtype=torch.int32),
                 work=torch.empty(nws, dtype=torch.uint8, device="cuda"))
        return None, t

    def run(o):
        ws.split_fc_fwd(X, W, bias, y, off, o["m"], o["s"], o["t"], o["work"])
        ws.combine_partials(o["m"].view(1, B), o["s"].view(1, B), o["t"].view(1, B), o["lse"], o["loss"], o["mean"])
        ws.split_fc_bwd(X, W, bias, o["lse"], y, off, -0.5, o["dX"], False, o["dW"], o["db"], o["work"])
        ws.split_fc_predict(X, W, bias, o["lse"], o["P"])
        ws.split_fc_top1(X, W, bias, off, o["top"], o["cls"], o["work"])
        torch.cuda.synchronize()

    _, plain = outputs(False)
    run(plain)
    guards, pitched = outputs(True)
    run(pitched)
    for name, g in guards.items():
        assert g.intact_outside_payload(), f"{tag}: bytes outside `{name}` were written"
    for name in plain:
        if name == "work":
            continue
        assert torch.equal(_bits(plain[name]), _bits(pitched[name])), f"{tag}: `{name}` differs with a pitch / guard bands"


def test_fused_sgd_writes_only_its_outputs(H):
    """The backward call that updates W and b in place: the weights sit in a pitched, guarded buffer."""
    import torch
    from paper_2011_09208_amd import binding as ws
    B, D, C = 513, 64, 23057
    p = inputs.make_inputs("guards-sgd", B, D, C, x_sigma=1.0, w_sigma=0.2, bias_sigma=0.5, seed=7)
    H.say(f"[guards] fused SGD: B={B} D={D} C={C}")
    X, W0 = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    b0 = torch.from_numpy(p.bias).cuda()
    y = torch.from_numpy(np.ascontiguousarray(p.labels, dtype=np.int32)).cuda()
    nws = max(ws.fwd_workspace_bytes(B, D, C), ws.bwd_workspace_bytes(B, D, C))
    m, s, t, lse, loss = (torch.empty(B, device="cuda") for _ in range(5))
    work = torch.empty(nws, dtype=torch.uint8, device="cuda")
    ws.split_fc_fwd(X, W0, b0, y, 0, m, s, t, work)
    ws.combine_partials(m.view(1, B), s.view(1, B), t.view(1, B), lse, loss, None)

    Wp, bp, dXp = W0.clone(), b0.clone(), torch.empty((B, D), device="cuda")
    ws.split_fc_bwd_sgd(X, Wp, bp, lse, y, 0, 1.0 / B, 0.5, dXp, False, work)
    gW, gb = Guarded(C, D, torch.bfloat16, pad_cols=8), Guarded(1, C, torch.float32)
    gX, gwork = Guarded(B, D, torch.float32, pad_cols=8), Guarded(1, nws, torch.uint8)
    gW.t.copy_(W0)
    gb.vec().copy_(b0)
    ws.split_fc_bwd_sgd(X, gW.t, gb.vec(), lse, y, 0, 1.0 / B, 0.5, gX.t, False, gwork.vec())
    torch.cuda.synchronize()
    for name, g in (("W", gW), ("b", gb), ("dX", gX), ("workspace", gwork)):
        assert g.intact_outside_payload(), f"bytes outside `{name}` were written"
    assert torch.equal(_bits(Wp), _bits(gW.t)) and torch.equal(_bits(bp), _bits(gb.vec()))
    assert torch.equal(_bits(dXp), _bits(gX.t))
    assert not torch.equal(_bits(Wp), _bits(W0))        # the update did something


def test_sp2_and_bridge_write_only_their_outputs(H):
    """The comparison path (partial logits, their reduction) and the two bridge-layer ends."""
    import torch
    from paper_2011_09208_amd import binding as ws
    B, D, C = 300, 256, 777
    p = inputs.make_inputs("guards-sp2", B, D, C, w_sigma=0.3, bias_sigma=0.8, seed=11)
    H.say(f"[guards] sp2 and bridge: B={B} D={D} C={C}")
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).cuda()
    y = torch.from_numpy(np.ascontiguousarray(p.labels, dtype=np.int32)).cuda()
    cuts = [0, 64, 256]
    Zg = [Guarded(B, C, torch.float32, pad_cols=(-C) % 4 + 4) for _ in cuts[1:]]
    Zp = [torch.empty((B, C + (-C) % 4), device="cuda")[:, :C] for _ in cuts[1:]]
    for zg, zp, a, e in zip(Zg, Zp, cuts[:-1], cuts[1:]):
        ws.sp2_partial_logits(X[:, a:e], W[:, a:e], zg.t)
        ws.sp2_partial_logits(X[:, a:e], W[:, a:e], zp)
    lse_g, loss_g = Guarded(1, B, torch.float32), Guarded(1, B, torch.float32)
    lse_p, loss_p = torch.empty(B, device="cuda"), torch.empty(B, device="cuda")
    ws.sp2_reduce_stats([z.t for z in Zg], bias, y, lse_g.vec(), loss_g.vec())
    ws.sp2_reduce_stats(Zp, bias, y, lse_p, loss_p)
    torch.cuda.synchronize()
    for name, g in [(f"Z_partial[{i}]", z) for i, z in enumerate(Zg)] + [("logsumexp", lse_g), ("loss", loss_g)]:
        assert g.intact_outside_payload(), f"bytes outside `{name}` were written"
    for zg, zp in zip(Zg, Zp):
        assert torch.equal(_bits(zg.t), _bits(zp))
    assert torch.equal(_bits(lse_g.vec()), _bits(lse_p)) and torch.equal(_bits(loss_g.vec()), _bits(loss_p))

    # bridge: gather uneven row blocks (features of the replicas), then reduce + partition gradient partials
    rows = [37, 0, 201, 62]
    blocks = [X[sum(rows[:i]): sum(rows[:i + 1])] for i in range(len(rows))]
    out = Guarded(B, D, torch.bfloat16, pad_cols=8)
    ws.bridge_gather(0, blocks, out.t)
    cols = [5, 1, 0, 7, 3]
    src = [X[:33, sum(cols[:i]): sum(cols[:i + 1])] for i in range(len(cols))]
    outc = Guarded(33, sum(cols), torch.bfloat16, pad_cols=1)
    ws.bridge_gather(1, src, outc.t)
    partials = [torch.randn((B, D), device="cuda", generator=torch.Generator(device="cuda").manual_seed(i)) for i in range(3)]
    parts = [Guarded(max(r, 1), D, torch.float32, pad_cols=4) for r in rows]
    ws.bridge_reduce_partition(partials, [g.t[:r] for g, r in zip(parts, rows)])
    torch.cuda.synchronize()
    assert out.intact_outside_payload() and outc.intact_outside_payload()
    assert torch.equal(_bits(out.t), _bits(X)) and torch.equal(_bits(outc.t), _bits(X[:33, :sum(cols)]))
    acc = (partials[0] + partials[1]) + partials[2]
    at = 0
    for g, r in zip(parts, rows):
        if r == 0:
            assert bool((g.raw == H.PATTERN).all())          # an empty part: nothing at all is written
        else:
            assert g.intact_outside_payload()
            assert torch.equal(_bits(g.t[:r]), _bits(acc[at:at + r]))
        at += r
