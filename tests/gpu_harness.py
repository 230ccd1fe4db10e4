"""Helpers for the GPU parity tests: run one training step of the split head through the
C-ABI binding, run the fp64 oracle on the same bits, and compare to the stated tolerances.
Not collected by pytest (no test_ prefix)."""
import json
import os
import sys

import numpy as np
import torch

from oracle import oracle
from paper_2011_09208_amd import inputs

# Tolerances of the parity gate (bf16 inputs, fp32 accumulation).
LOSS_REL = 1e-3
LSE_ABS = 2e-3
GRAD_REL_TO_MAX = 2e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def record(tag, shape, rep):
    """Appends the achieved errors of one parity case to the file named by WS_PARITY_LOG (one JSON object
    per line), so that a run of the suite leaves the margins behind and not only pass/fail."""
    path = os.environ.get("WS_PARITY_LOG")
    if not path:
        return
    with open(path, "a") as f:
        f.write(json.dumps({"case": tag, "shape": shape, **{k: float(v) for k, v in rep.items()}}) + "\n")


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return inputs.bf16_bits_to_f64(t.view(torch.int16).cpu().numpy().view(np.uint16))


def run_step(X_bits, W_bits, bias, labels, shards, g=1.0, w_lo=0, want_db=True, loss_mean=False,
             lse_override=None, keep_dW=None):
    """fwd on every shard -> combine -> bwd on every shard (dX accumulated across shards).

    W_bits holds classes [w_lo, w_lo + rows); `shards` = [(class_offset, C_shard)].
    Returns numpy arrays: per-shard m, s, t [S, B]; lse, loss [B]; dX [B, D];
    dW list of [C_s, D] (float64 upcast of bf16), db list of [C_s].
    `lse_override` [B] replaces the combined log-sum-exp as the backward call's input (used when only
    some shards of a wider layer are evaluated).  `keep_dW` = indices of the shards whose dW is copied back
    (default all; the others give None: dW of a very wide layer is gigabytes on the host).
    """
    from paper_2011_09208_amd import binding as ws

    X = dev_bf16(X_bits)
    W = dev_bf16(W_bits)
    B, D = X.shape
    y = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).cuda()
    b_dev = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).cuda()
    S = len(shards)
    m = torch.full((S, B), float("nan"), device="cuda")
    s = torch.full((S, B), float("nan"), device="cuda")
    t = torch.full((S, B), float("nan"), device="cuda")
    lse = torch.full((B,), float("nan"), device="cuda")
    loss = torch.full((B,), float("nan"), device="cuda")
    mean = torch.full((1,), float("nan"), device="cuda") if loss_mean else None
    fwd_ws = max(ws.fwd_workspace_bytes(B, D, c) for _, c in shards)
    bwd_ws = max(ws.bwd_workspace_bytes(B, D, c) for _, c in shards)
    work = torch.empty(max(fwd_ws, bwd_ws), dtype=torch.uint8, device="cuda")
    work.fill_(0xFF)       # NaN patterns: stale workspace must never leak into a result
    for i, (off, c) in enumerate(shards):
        Ws = W[off - w_lo: off - w_lo + c]
        bs = None if b_dev is None else b_dev[off - w_lo: off - w_lo + c]
        ws.split_fc_fwd(X, Ws, bs, y, off, m[i], s[i], t[i], work)
    ws.combine_partials(m, s, t, lse, loss, mean)
    lse_bwd = lse if lse_override is None else torch.from_numpy(
        np.ascontiguousarray(lse_override, dtype=np.float32)).cuda()
    dX = torch.full((B, D), float("nan"), device="cuda")
    dWs, dbs = [], []
    for i, (off, c) in enumerate(shards):
        Ws = W[off - w_lo: off - w_lo + c]
        bs = None if b_dev is None else b_dev[off - w_lo: off - w_lo + c]
        dW = torch.full((c, D), float("nan"), device="cuda", dtype=torch.bfloat16)
        db = torch.full((c,), float("nan"), device="cuda") if want_db else None
        ws.split_fc_bwd(X, Ws, bs, lse_bwd, y, off, g, dX, i > 0, dW, db, work)
        dWs.append(dW)
        dbs.append(db)
    torch.cuda.synchronize()
    out = dict(m=m.cpu().numpy(), s=s.cpu().numpy(), t=t.cpu().numpy(), lse=lse.cpu().numpy(),
               loss=loss.cpu().numpy(), dX=dX.cpu().numpy(),
               dW=[bf16_to_f64(w) if keep_dW is None or i in keep_dW else None for i, w in enumerate(dWs)],
               db=[None if d is None else d.cpu().numpy() for d in dbs])
    if loss_mean:
        out["loss_mean"] = float(mean.cpu().numpy()[0])
    return out


def oracle_step(X_bits, W_bits, bias, labels, shards, g=1.0, w_lo=0):
    """The same step by the oracle: unsharded result over the union of the shards plus per-shard statistics.
    The shards must tile a contiguous class range that starts at w_lo."""
    X = inputs.bf16_bits_to_f64(X_bits)
    W = inputs.bf16_bits_to_f64(W_bits)
    b = None if bias is None else np.asarray(bias, dtype=np.float64)
    y = np.asarray(labels, dtype=np.int64)
    ms, ss, ts = [], [], []
    for off, c in shards:
        sl = slice(off - w_lo, off - w_lo + c)
        mm, sss, tt = oracle.partials(X, W[sl], None if b is None else b[sl], y, off)
        ms.append(mm), ss.append(sss), ts.append(tt)
    lse, loss = oracle.combine(ms, ss, ts)
    dX = np.zeros_like(X)
    dWs, dbs = [], []
    for off, c in shards:
        sl = slice(off - w_lo, off - w_lo + c)
        gr = oracle.shard_grads(X, W[sl], None if b is None else b[sl], lse, y, off, g)
        dX += gr["dX_partial"]
        dWs.append(gr["dW"])
        dbs.append(gr["db"])
    return dict(m=np.stack(ms), s=np.stack(ss), t=np.stack(ts), lse=lse, loss=loss, dX=dX, dW=dWs, db=dbs)


def max_rel_to_max(got, ref):
    scale = np.max(np.abs(ref))
    if scale == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / scale)


def compare(got, ref, labels, shards, tag="", gate="stated"):
    """Asserts the parity gate; returns a dict of the error figures.

    gate="stated" (the workload configurations): exactly the stated tolerances, nothing added: loss
    relative error <= 1e-3 per row, log-sum-exp / row max / label logit absolute error <= 2e-3.
    gate="fp32_floor" (random ragged shapes, where a row's loss can be ~0 when its label happens to be the
    arg-max): the same absolute gates; the per-row loss gate gets an absolute floor of 16 * 2^-24 * |z|max,
    the rounding that lse and the label logit carry as fp32 numbers before they are subtracted.
    gate="large_logits" (the stress cases with |z| of a few hundred): the absolute gates are multiplied by
    max(1, |z|max), since the fp32 logits themselves are only known to |z| * 2^-24 * (summation error).
    Every gradient must be within 2e-2 of its largest magnitude in all three."""
    assert gate in ("stated", "fp32_floor", "large_logits")
    y = np.asarray(labels, dtype=np.int64)
    rep = {}
    for k in ("m", "s", "t", "lse", "loss", "dX"):
        assert np.all(np.isfinite(got[k])), f"{tag}: non-finite values in {k}"
    # integer part: label logit is exactly zero outside the shard and owned by exactly one shard
    for i, (off, c) in enumerate(shards):
        inside = (y >= off) & (y < off + c)
        assert np.all(got["t"][i][~inside] == 0.0), f"{tag}: label_logit not exactly 0 outside shard {i}"
    rep["row_max_abs"] = float(np.max(np.abs(got["m"] - ref["m"])))
    rep["sumexp_rel"] = float(np.max(np.abs(got["s"] - ref["s"]) / ref["s"]))
    rep["label_logit_abs"] = float(np.max(np.abs(got["t"] - ref["t"])))
    rep["lse_abs"] = float(np.max(np.abs(got["lse"] - ref["lse"])))
    rep["loss_rel"] = float(np.max(np.abs(got["loss"] - ref["loss"]) / np.maximum(np.abs(ref["loss"]), 1e-30)))
    rep["loss_abs"] = float(np.max(np.abs(got["loss"] - ref["loss"])))
    zmax = float(np.max(np.abs(ref["m"])))
    zscale = max(1.0, zmax) if gate == "large_logits" else 1.0
    assert rep["row_max_abs"] <= LSE_ABS * zscale, (tag, rep)
    assert rep["sumexp_rel"] <= 1e-3 + (LSE_ABS * zscale if gate == "large_logits" else 0.0), (tag, rep)
    assert rep["label_logit_abs"] <= LSE_ABS * zscale, (tag, rep)
    assert rep["lse_abs"] <= LSE_ABS * zscale, (tag, rep)
    floor = {"stated": 0.0, "fp32_floor": 16.0 * 2.0 ** -24 * max(1.0, zmax), "large_logits": LSE_ABS * zscale * 1e-1}[gate]
    ok = np.abs(got["loss"] - ref["loss"]) <= LOSS_REL * np.abs(ref["loss"]) + floor
    assert np.all(ok), (tag, rep)
    rep["dX"] = max_rel_to_max(got["dX"], ref["dX"])
    assert rep["dX"] <= GRAD_REL_TO_MAX, (tag, rep)
    rep["dW"], rep["db"] = 0.0, 0.0
    wscale = max(np.max(np.abs(w)) for w in ref["dW"]) or 1.0     # a one-class layer has zero gradients
    bscale = max(np.max(np.abs(d)) for d in ref["db"]) or 1.0
    for i in range(len(shards)):
        if got["dW"][i] is not None:
            assert np.all(np.isfinite(got["dW"][i])), f"{tag}: non-finite dW in shard {i}"
            rep["dW"] = max(rep["dW"], float(np.max(np.abs(got["dW"][i] - ref["dW"][i])) / wscale))
        if got["db"][i] is not None:
            assert np.all(np.isfinite(got["db"][i])), f"{tag}: non-finite db in shard {i}"
            rep["db"] = max(rep["db"], float(np.max(np.abs(got["db"][i] - ref["db"][i])) / bscale))
    assert rep["dW"] <= GRAD_REL_TO_MAX, (tag, rep)
    assert rep["db"] <= GRAD_REL_TO_MAX, (tag, rep)
    return rep


PATTERN = 0xA5
GUARD = 8192          # bytes before and after every payload


class Guarded:
    """rows x cols elements of `dtype` with a row pitch of cols + pad_cols, guard bytes around them."""

    def __init__(self, rows, cols, dtype, pad_cols=0, device="cuda"):
        self.rows, self.cols, self.pitch, self.dtype = rows, cols, cols + pad_cols, dtype
        self.es = torch.empty((), dtype=dtype).element_size()
        self.nbytes = rows * self.pitch * self.es
        self.raw = torch.full((GUARD + self.nbytes + GUARD,), PATTERN, dtype=torch.uint8, device=device)
        self.t = self._payload(self.raw, dtype)

    def _payload(self, raw, dtype):
        return raw[GUARD:GUARD + self.nbytes].view(dtype).view(self.rows, self.pitch)[:, :self.cols]

    def vec(self):
        assert self.rows == 1
        return self.t[0]

    def intact_outside_payload(self):
        r = self.raw.clone()
        as_int = {1: torch.uint8, 2: torch.int16, 4: torch.int32}[self.es]
        fill = {1: PATTERN, 2: int(np.int16(np.uint16(0xA5A5))), 4: int(np.int32(np.uint32(0xA5A5A5A5)))}[self.es]
        self._payload(r, as_int).fill_(fill)
        return bool((r == PATTERN).all())
