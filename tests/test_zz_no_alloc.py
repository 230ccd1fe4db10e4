"""The forward entry point that allocates nothing (ws_split_fc_fwd_static): its output against the
workspace-taking entry point's, bit for bit (same kernels), and against the fp64 oracle to the stated gate,
on two calls in a row, the second with a smaller input (the built-in scratch keeps the first call's
contents)."""
import gc

import numpy as np
import pytest

from paper_2011_09208_amd import inputs

pytestmark = pytest.mark.gpu


def _one_call(H, ws, torch, B, D, C, off, seed):
    from oracle import oracle
    p = inputs.make_inputs("static", B, D, C, x_sigma=1.0, w_sigma=0.2, bias_sigma=1.0, seed=seed)
    labels = (p.labels.astype(np.int64) + off - C // 3).astype(np.int32)     # some labels fall outside the shard
    H.say(f"[no-alloc] ws_split_fc_fwd_static B={B} D={D} C_shard={C} class_offset={off}")
    dev = torch.device("cuda")
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    bias = torch.from_numpy(p.bias).to(dev)
    y = torch.from_numpy(labels).to(dev)
    ref_out = [torch.full((B,), float("nan"), device=dev) for _ in range(3)]
    work = torch.empty(ws.fwd_workspace_bytes(B, D, C), dtype=torch.uint8, device=dev)
    ws.split_fc_fwd(X, W, bias, y, off, *ref_out, work)
    got = [torch.full((B,), float("nan"), device=dev) for _ in range(3)]
    # nothing may be allocated by the call: neither through torch (count of its allocator's allocations; tensors of
    # earlier tests may be freed at any time, so not the bytes in use) nor behind its back (the device's free memory)
    gc.collect()
    torch.cuda.synchronize()
    n_alloc = torch.cuda.memory_stats()["allocation.all.allocated"]
    free_before = torch.cuda.mem_get_info()[0]
    ws.split_fc_fwd_static(X, W, bias, y, off, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == n_alloc
    assert torch.cuda.mem_get_info()[0] >= free_before
    for g, r in zip(got, ref_out):
        assert torch.equal(g.view(torch.int32), r.view(torch.int32))
    m, s, t = oracle.partials(inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits),
                              p.bias.astype(np.float64), labels, off)
    gm, gs, gt = (g.cpu().numpy() for g in got)
    assert np.max(np.abs(gm - m)) <= H.LSE_ABS and np.max(np.abs(gt - t)) <= H.LSE_ABS
    assert np.max(np.abs(gs - s) / s) <= 1e-3
    inside = (labels >= off) & (labels < off + C)
    assert 0 < inside.sum() < B and np.all(gt[~inside] == 0.0)


def test_static_scratch_forward_two_calls_second_smaller():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU; there is no CPU fallback")
    from tests import gpu_harness as H
    from paper_2011_09208_amd import binding as ws
    _one_call(H, ws, torch, 1100, 128, 14000, 5000, seed=1)      # 275 tiles: full and thin, 1.4 MB of scratch
    _one_call(H, ws, torch, 300, 64, 1000, 700, seed=2)          # smaller: thin tiles only, stale partials around it
    # beyond the built-in scratch: refused on the host, nothing launched
    B, D, C = 8192, 64, 600_000
    assert ws.fwd_workspace_bytes(B, D, C) > ws.STATIC_SCRATCH_BYTES
    X = torch.empty((B, D), device="cuda", dtype=torch.bfloat16)
    W = torch.empty((C, D), device="cuda", dtype=torch.bfloat16)
    y = torch.zeros(B, device="cuda", dtype=torch.int32)
    out = [torch.zeros(B, device="cuda") for _ in range(3)]
    with pytest.raises(ws.WhaleSplitError) as e:
        ws.split_fc_fwd_static(X, W, None, y, 0, *out)
    assert str(e.value) == "WS_ERR_LIMIT"
