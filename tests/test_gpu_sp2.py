"""GPU parity of the contraction-split comparison path (SP2 of Section 3.2.2) through the C-ABI binding:
partial logits of every slice and the reduced log-sum-exp / loss against the fp64 oracle."""
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


def _sp2_parity(H, p, cuts, tag):
    import torch
    from oracle import oracle
    from paper_2011_09208_amd import binding as ws
    H.say(f"[parity] {tag}: B={p.B} D={p.D} C={p.C} contraction cuts {cuts}")
    X, W = H.dev_bf16(p.X_bits), H.dev_bf16(p.W_bits)
    X64, W64 = inputs.bf16_bits_to_f64(p.X_bits), inputs.bf16_bits_to_f64(p.W_bits)
    b64 = None if p.bias is None else p.bias.astype(np.float64)
    bias = None if p.bias is None else torch.from_numpy(p.bias).cuda()
    y = torch.from_numpy(p.labels.astype(np.int32)).cuda()
    ldz = (p.C + 3) // 4 * 4
    parts = []
    ref_sum = np.zeros((p.B, p.C))
    worst = 0.0
    for a, e in zip(cuts[:-1], cuts[1:]):
        Zb = torch.full((p.B, ldz), float("nan"), device="cuda")
        ws.sp2_partial_logits(X[:, a:e], W[:, a:e], Zb[:, :p.C])
        torch.cuda.synchronize()
        ref = oracle.sp2_partial_logits(X64, W64, a, e)
        got = Zb[:, :p.C].cpu().numpy()
        scale = max(1.0, float(np.max(np.abs(ref))))
        err = float(np.max(np.abs(got - ref)))
        assert err <= H.LSE_ABS * scale, (tag, a, e, err)
        if ldz > p.C:
            assert bool(torch.isnan(Zb[:, p.C:]).all())
        worst = max(worst, err)
        ref_sum += ref
        parts.append(Zb[:, :p.C])
    lse = torch.full((p.B,), float("nan"), device="cuda")
    loss = torch.full((p.B,), float("nan"), device="cuda")
    ws.sp2_reduce_stats(parts, bias, y, lse, loss)
    torch.cuda.synchronize()
    # the oracle's reduction of the ORACLE's partials (independent of the GPU's)
    ref_parts = [oracle.sp2_partial_logits(X64, W64, a, e) for a, e in zip(cuts[:-1], cuts[1:])] if p.B * p.C < 5e6 \
        else [ref_sum]
    rl, ro = oracle.sp2_reduce(ref_parts, b64, p.labels.astype(np.int64))
    zscale = max(1.0, float(np.max(np.abs(ref_sum))))
    gl, go = lse.cpu().numpy(), loss.cpu().numpy()
    assert np.max(np.abs(gl - rl)) <= H.LSE_ABS * zscale
    assert np.all(np.abs(go - ro) <= H.LOSS_REL * np.abs(ro) + H.LSE_ABS * zscale * 1e-1)
    H.say(f"[parity] {tag}: partial logits max abs err {worst:.2e}, lse {np.max(np.abs(gl - rl)):.2e}, "
          f"loss rel {np.max(np.abs(go - ro) / np.maximum(np.abs(ro), 1e-30)):.2e}")


def test_sp2_small_and_ragged(H):
    p = inputs.make_config("cfg1")
    _sp2_parity(H, p, [0, 64, 256], "sp2 cfg1")
    q = inputs.make_inputs("sp2", 300, 256, 777, w_sigma=0.3, bias_sigma=0.8, seed=51)
    _sp2_parity(H, q, [0, 64, 128, 256], "sp2 ragged")
    r = inputs.make_inputs("sp2", 257, 128, 1030, w_sigma=0.3, bias_sigma=0.8, seed=52)
    _sp2_parity(H, r, [0, 128], "sp2 one slice")


def test_sp2_full_size(H):
    """The paper's comparison shape (100K classes): B = 1024, D = 2048 cut 8 ways, C = 100 000."""
    p = inputs.make_config("headline")
    _sp2_parity(H, p, list(range(0, 2049, 256)), "sp2 headline")
