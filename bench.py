#!/usr/bin/env python3
"""Benchmark of the split fully-connected + softmax head on one MI355X.

One step = the whole hot path over one synthetic batch: split_fc_fwd on every shard ->
combine_partials -> split_fc_bwd on every shard, through the C-ABI library, inputs resident
in HBM.  Workload: the paper's motivating classifier at the headline shape (B = 1024 rows,
D = 2048 features, C = 100 000 classes as one shard; Section 1, Section 2.1).

Prints ONE JSON line: samples/s for fwd+bwd, the MFMA roofline of the slowest GEMM kernel
(algorithmic flops per launch / average launch time from HIP events recorded on the launch
stream inside the timed region), the per-kernel breakdown, and the fp64 oracle timed on the
host cores as a CPU baseline.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_DENSE_PEAK_TFLOPS = 2516.6      # 256 CUs x 2.4 GHz x 4096 flop/clk/CU
HBM_PEAK_GBS = 8000.0
GEMM_KERNELS = ("fwd_logits_stats", "bwd_recompute_dz", "bwd_dx", "bwd_dw")


def read_traffic(workload):
    """HBM bytes per launch of every kernel from the committed rocprofv3 --pmc summary of this workload, and
    the library version that summary was taken with (counters need a profiler run of their own, so the
    figure cannot be measured inside this program)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return {}, None
    out, version = {}, None
    with open(path) as f:
        for line in f:
            parts = line.split()
            if len(parts) >= 2 and parts[0].startswith("traffic_bytes:"):
                out[parts[0].split(":", 1)[1]] = float(parts[1])
            if len(parts) >= 2 and parts[0] == "library_version:":
                version = int(parts[1])
    return out, version


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements outside the timed step (bridge ends, SP1 vs SP2 forward)")
    ap.add_argument("--sustain-seconds", type=float, default=2.0,
                    help="after the timed steps, keep stepping for about this long and report the step time "
                         "of that loop as `sustained` (0 = skip)")
    ap.add_argument("--ceiling", action="store_true",
                    help="instead of the step, measure what the machine allows the GEMM main loop: an MFMA-only "
                         "loop and the library's main loop as a plain GEMM, on constant and on random operands, "
                         "with torch.matmul beside them as context; prints one JSON line")
    ap.add_argument("--trace-dw", action="store_true",
                    help="instead of timing the step, run it with the instrumented copy of the dW kernel and print "
                         "where a workgroup's cycles go (per-tile shader-clock stamps), one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (one shard per call, shards run one after another); "
                 "--gpus must be 1")

    import numpy as np
    import torch
    from paper_2011_09208_amd import inputs
    from paper_2011_09208_amd import binding as ws      # raises if the HIP library is not built

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU fallback")
    if args.ceiling:
        print(json.dumps(measure_ceiling(ws, torch)), flush=True)
        return

    # cfg5 and million time their first shard only (50 000 of 400 000, 125 000 of 1 000 000 classes);
    # the other rows of W are not kept
    first_shard_only = {"cfg5": 50_000, "million": 125_000}
    p = inputs.make_config(args.workload, w_rows=first_shard_only.get(args.workload))
    B, D = p.B, p.D
    shards = p.shards if args.workload not in first_shard_only else p.shards[:1]
    C = p.W_bits.shape[0]
    dev = torch.device("cuda:0")
    X = torch.from_numpy(p.X_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    W = torch.from_numpy(p.W_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    y = torch.from_numpy(p.labels).to(dev)
    S = len(shards)
    m = torch.empty((S, B), device=dev)
    s = torch.empty((S, B), device=dev)
    t = torch.empty((S, B), device=dev)
    lse = torch.empty(B, device=dev)
    loss = torch.empty(B, device=dev)
    dX = torch.empty((B, D), device=dev)
    dW = torch.empty((W.shape[0], D), device=dev, dtype=torch.bfloat16)
    db = torch.empty(W.shape[0], device=dev)
    nbytes = max(max(ws.fwd_workspace_bytes(B, D, c), ws.bwd_workspace_bytes(B, D, c)) for _, c in shards)
    work = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def step():
        for i, (off, c) in enumerate(shards):
            ws.split_fc_fwd(X, W[off:off + c], None, y, off, m[i], s[i], t[i], work)
        ws.combine_partials(m, s, t, lse, loss, None)
        for i, (off, c) in enumerate(shards):
            ws.split_fc_bwd(X, W[off:off + c], None, lse, y, off, 1.0, dX, i > 0, dW[off:off + c],
                            db[off:off + c], work)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)        # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.trace_dw:
        print(json.dumps(trace_dw(ws, torch, np, step, args.workload, B, D, shards)), flush=True)
        return

    sustained = None
    if args.sustain_seconds > 0:
        # The part is power-limited and its clocks take a while to settle: keep stepping for about two seconds
        # (the rate after seconds at load, reported as `sustained`); the K timed steps below then start on a
        # chip in that steady state instead of one that has just come out of idle.
        probe0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        est_ms = max((time.perf_counter() - probe0) * 1e3, 1e-2)
        n = max(args.steps, int(args.sustain_seconds * 1e3 / est_ms) + 1)
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        sustained = {"ms_per_step": round(dt * 1e3 / n, 4), "steps": n, "seconds": round(dt, 2),
                     "value": round(B * n / dt, 1), "unit": "samples/s"}

    # untimed-by-events run first: the wall-clock figure without any event records in the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    plain_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # the timed region proper: in about five of its steps, evenly spaced, each kernel launch is bracketed by HIP
    # events on its stream (a pair of records costs about as much as one of the small kernels, so not in every step)
    EVENT_EVERY = max(4, args.steps // 5)
    ws.profile_enable((args.steps // EVENT_EVERY + 1) * (7 * S + 2) + 16)
    ws.profile_reset()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        ws.profile_pause(i % EVENT_EVERY != 0)
        step()
    marks[args.steps].record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = ws.profile_read()
    ws.profile_enable(0)

    c_total = sum(c for _, c in shards)
    timed_steps = len(range(0, args.steps, EVENT_EVERY))
    kernels = {}
    for name, (tot_ms, n) in prof.items():
        avg = tot_ms / n
        kernels[name] = {"avg_ms": round(avg, 5), "launches_per_step": n / timed_steps, "timed_launches": n}
    # each GEMM kernel launch performs 2 * B * D * C_shard flops; with several shards take the mean launch
    flops_per_launch = 2.0 * B * D * c_total / S
    dominant = max(GEMM_KERNELS, key=lambda k: kernels[k]["avg_ms"])
    for k in GEMM_KERNELS:
        kernels[k]["tflops"] = round(flops_per_launch / (kernels[k]["avg_ms"] * 1e-3) / 1e12, 2)
    # the two reduction kernels of the forward path move a few MB: HBM GB/s from their algorithmic bytes
    n_ct = -(-(c_total // S) // 256)
    small_bytes = {"merge_class_tiles": 8.0 * n_ct * (-(-B // 256) * 256) + 8.0 * B,
                   "combine_partials": 12.0 * S * B + 8.0 * B}
    for k, nbytes_k in small_bytes.items():
        if k in kernels:
            kernels[k]["GB/s"] = round(nbytes_k / (kernels[k]["avg_ms"] * 1e-3) / 1e9, 1)
    achieved = kernels[dominant]["tflops"]
    traffic_table, traffic_version = read_traffic(args.workload)
    traffic = traffic_table.get(dominant) if traffic_version == ws.version() else None
    traffic_source = (f"profiles/hbm_traffic_{args.workload}.txt, rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of library "
                      f"version {traffic_version}" if traffic is not None else
                      f"none for library version {ws.version()} and this workload (counters need their own profiler run)")
    credited = 6.0 * B * D * c_total
    value = B / (ms_per_step * 1e-3)
    # Algorithmic HBM bytes of one launch of each GEMM kernel (operands read once, outputs written once).
    cs = c_total / S
    cpad = -(-cs // 256) * 256
    bpad = -(-B // 256) * 256
    alg_bytes = {
        "fwd_logits_stats": 2 * D * cs + 2 * B * D + 8 * bpad * (cpad / 256),
        "bwd_recompute_dz": 2 * D * cs + 2 * B * D + 2 * bpad * cpad + 2 * D * bpad,
        "bwd_dx": 2 * bpad * cpad + 2 * D * cs + 4 * B * D,
        "bwd_dw": 2 * bpad * cpad + 2 * D * bpad + 2 * D * cs,
    }
    # a kernel whose flops per algorithmic byte fall below the machine balance is bound by HBM, not MFMA
    balance = BF16_DENSE_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if flops_per_launch / alg_bytes[dominant] < balance:
        gbs = alg_bytes[dominant] / (kernels[dominant]["avg_ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "traffic_source": traffic_source}
    else:
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": achieved, "peak": BF16_DENSE_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / BF16_DENSE_PEAK_TFLOPS, 4), "traffic": traffic,
                    "traffic_source": traffic_source}

    result = {
        "metric": "split-FC fwd+bwd samples/sec at D=2048,C=100K,B=1024; % bf16 MFMA peak",
        "value": round(value, 1),
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={B} D={D} C={C} shards={S} (fwd all shards -> combine -> bwd all shards)"},
        "pct_bf16_mfma_peak_credited_6BDC": round(100.0 * credited / (ms_per_step * 1e-3) / (BF16_DENSE_PEAK_TFLOPS * 1e12), 2),
        "pct_bf16_mfma_peak_executed_8BDC": round(100.0 * credited * 8 / 6 / (ms_per_step * 1e-3) / (BF16_DENSE_PEAK_TFLOPS * 1e12), 2),
        "ms_per_step_without_event_records": round(plain_ms, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
        "ms_per_step_min": round(per_step[0], 4),
        "roofline": roofline,
        "kernels": kernels,
    }
    if sustained is not None:
        sustained["pct_bf16_mfma_peak_credited_6BDC"] = round(
            100.0 * credited / (sustained["ms_per_step"] * 1e-3) / (BF16_DENSE_PEAK_TFLOPS * 1e12), 2)
        result["sustained"] = sustained

    if not args.no_extras:
        measure_extras(args, result, ws, torch, dev, X, W, y, B, D, C, work, lse, loss)

    if not args.no_cpu_baseline and args.workload not in first_shard_only:   # one shard of W only: no unsharded oracle
        cpu_baseline(args, result, inputs, p, B, D, C, lse)
    print(json.dumps(result), flush=True)


def measure_extras(args, result, ws, torch, dev, X, W, y, B, D, C, work, lse, loss):
    """Measurements outside the timed step.  The bridge-layer ends at this workload's shape (8 replicas feed X;
    8 shards' dX_partial go back): HBM-bound copy / add kernels, timed with events on the launch stream."""
    R = 8 if B % 8 == 0 else 1
    blocks = [X[i * (B // R):(i + 1) * (B // R)].clone() for i in range(R)]
    Xg = torch.empty_like(X)
    partials = [torch.randn((B, D), device=dev) for _ in range(8)]
    outs = [torch.empty((B // R, D), device=dev) for _ in range(R)]

    def timed(fn, iters=50):
        for _ in range(5):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    # arguments marshalled once: at these sizes a call is a few microseconds of GPU time
    g_args = ws.bridge_gather_args(0, blocks, Xg)
    r_args = ws.bridge_reduce_partition_args(partials, outs)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    g_us = timed(lambda: ws.lib.ws_bridge_gather(*g_args, stream))
    r_us = timed(lambda: ws.lib.ws_bridge_reduce_partition(*r_args, stream))
    g_bytes, r_bytes = 2.0 * B * D * 2, (len(partials) + 1.0) * B * D * 4
    result["bridge"] = {
        "gather": {"us": round(g_us, 2), "bytes": g_bytes, "GB/s": round(g_bytes / g_us / 1e3, 1)},
        "reduce_partition": {"us": round(r_us, 2), "bytes": r_bytes, "GB/s": round(r_bytes / r_us / 1e3, 1)},
        "bound": "hbm", "peak_GB/s": HBM_PEAK_GBS,
        "shape": f"{R} replica blocks of [{B // R}, {D}] bf16 -> X; {len(partials)} fp32 [B, D] partials -> {R} blocks",
    }
    del blocks, Xg, partials, outs

    # The backward call with the SGD update folded in (W and dW are both bf16: same bytes written, W read
    # once more), against the plain one, on the timed workload's first shard.  lr = 0 keeps W as it is.
    if work.numel() >= ws.bwd_workspace_bytes(B, D, W.shape[0]):       # single-shard workloads
        dXs = torch.empty((B, D), device=dev)
        dWs = torch.empty((W.shape[0], D), device=dev, dtype=torch.bfloat16)
        plain_us = timed(lambda: ws.split_fc_bwd(X, W, None, lse, y, 0, 1.0, dXs, False, dWs, None, work), 10)
        fused_us = timed(lambda: ws.split_fc_bwd_sgd(X, W, None, lse, y, 0, 1.0, 0.0, dXs, False, work), 10)
        result["fused_sgd_backward"] = {"bwd_ms": round(plain_us / 1e3, 4), "bwd_sgd_ms": round(fused_us / 1e3, 4),
                                        "shape": f"B={B} D={D} C_shard={W.shape[0]}"}
        del dXs, dWs

    # Context only (never the product path): the vendor GEMM library, through torch.matmul, on the three GEMM
    # shapes of this step with the same operands (bf16 in, bf16 out).
    if args.workload == "headline":
        Zt = torch.empty((B, C), device=dev, dtype=torch.bfloat16)
        dZt = (torch.randn((B, C), device=dev) * 1e-5).to(torch.bfloat16)
        dXt = torch.empty((B, D), device=dev, dtype=torch.bfloat16)
        dWt = torch.empty((C, D), device=dev, dtype=torch.bfloat16)
        fl = 2.0 * B * D * C
        ctx = {}
        for name, fn in (("logits = X . W^T", lambda: torch.matmul(X, W.t(), out=Zt)),
                         ("dX = dz . W", lambda: torch.matmul(dZt, W, out=dXt)),
                         ("dW = dz^T . X", lambda: torch.matmul(dZt.t(), X, out=dWt))):
            us = timed(fn, 10)
            ctx[name] = {"ms": round(us / 1e3, 4), "tflops": round(fl / us / 1e6, 1)}
        result["context_torch_matmul_bf16"] = ctx
        del Zt, dZt, dXt, dWt

    # Forward pass of the layer under the paper's two sharding patterns (Section 5.3.2), 8 ways, every
    # device's share run one after another on this GPU: SP1 = 8 class shards (fwd + combine), SP2 = 8
    # contraction slices (partial logits over all classes, then the reduction an AllReduce would do).
    if args.workload == "headline":
        ways = 8
        cw, dw_ = C // ways, D // ways
        m8, s8, t8 = (torch.empty((ways, B), device=dev) for _ in range(3))
        zparts = [torch.empty((B, C), device=dev) for _ in range(ways)]
        lse1, loss1 = torch.empty(B, device=dev), torch.empty(B, device=dev)
        lse2, loss2 = torch.empty(B, device=dev), torch.empty(B, device=dev)

        def sp1_fwd():
            for i in range(ways):
                ws.split_fc_fwd(X, W[i * cw:(i + 1) * cw], None, y, i * cw, m8[i], s8[i], t8[i], work)
            ws.combine_partials(m8, s8, t8, lse1, loss1, None)

        def sp2_fwd():
            for i in range(ways):
                ws.sp2_partial_logits(X[:, i * dw_:(i + 1) * dw_], W[:, i * dw_:(i + 1) * dw_], zparts[i])
            ws.sp2_reduce_stats(zparts, None, y, lse2, loss2)

        sp1_us, sp2_us = timed(sp1_fwd, 10), timed(sp2_fwd, 10)
        result["sharding_patterns_forward"] = {
            "ways": ways, "sp1_ms": round(sp1_us / 1e3, 4), "sp2_ms": round(sp2_us / 1e3, 4),
            "sp2_over_sp1": round(sp2_us / sp1_us, 2),
            "sp2_partial_logit_bytes_written_and_read": 2.0 * ways * B * C * 4,
            "sp1_exchanged_bytes": 12.0 * ways * B,
            "max_abs_lse_diff_sp1_vs_sp2": float((lse1 - lse2).abs().max()),
            "max_abs_lse_diff_sp1_vs_one_shard": float((lse1 - lse).abs().max()),
        }
        del zparts


def trace_dw(ws, torch, np, step, workload, B, D, shards):
    """Where the cycles of a dW workgroup go: the step is run with the instrumented copy of the kernel (same
    arithmetic and stores; thread 0 of every workgroup stamps the shader clock at six points and notes its compute
    unit).  The trace kept is the one of the last shard's launch of the last step."""
    n_dt = D // 256
    tiles = max(n_dt * -(-c // 256) for _, c in shards)
    trace = torch.zeros((tiles, 8), dtype=torch.int64, device="cuda:0")
    for _ in range(20):
        step()
    torch.cuda.synchronize()
    ws.profile_trace_dw(trace)
    try:
        for _ in range(5):
            step()
        torch.cuda.synchronize()
    finally:
        ws.profile_trace_dw(None)
    n = n_dt * -(-shards[-1][1] // 256)
    tr = trace[:n].cpu().numpy()
    tr = tr[tr[:, 0] > 0]            # tiles of a last round that ran as thin tiles are not traced
    names = ["entry -> main loop starts", "main loop (%d k-steps)" % (-(-B // 64)), "accumulators -> LDS tile, barrier",
             "row stores issued", "row stores acknowledged"]
    ph = np.diff(tr[:, :6], axis=1)
    phases = [{"phase": nm, "mean": round(float(ph[:, i].mean()), 1), "median": float(np.median(ph[:, i])),
               "p90": float(np.percentile(ph[:, i], 90))} for i, nm in enumerate(names)]
    total = tr[:, 5] - tr[:, 0]
    # HW_ID: compute unit bits 8-11, shader array bit 12, shader engine bits 13-15; XCC_ID in the upper word
    hw = tr[:, 7]
    unit = (hw >> 32) * 4096 + ((hw >> 8) & 0xff)
    gaps, per_unit, busy = [], [], []
    for u in np.unique(unit):
        rows = tr[unit == u]
        rows = rows[np.argsort(rows[:, 0])]
        per_unit.append(len(rows))
        gaps.extend((rows[1:, 0] - rows[:-1, 5]).tolist())
        busy.append(int(rows[-1, 5] - rows[0, 0]))
    gaps = np.array(gaps if gaps else [0])
    return {"what": "dW kernel, per-tile shader-clock stamps of thread 0 (cycles)", "workload": workload,
            "library_version": ws.version(), "tiles": int(n), "tiles_traced": int(len(tr)), "phases": phases,
            "tile_total": {"mean": round(float(total.mean()), 1), "median": float(np.median(total))},
            "compute_units_seen": int(len(per_unit)),
            "tiles_per_unit": {"min": int(min(per_unit)), "mean": round(float(np.mean(per_unit)), 2), "max": int(max(per_unit))},
            "gap_between_tiles_on_a_unit": {"mean": round(float(gaps.mean()), 1), "median": float(np.median(gaps)),
                                            "p90": float(np.percentile(gaps, 90))},
            "unit_first_entry_to_last_ack": {"mean": round(float(np.mean(busy)), 1), "max": int(max(busy))}}


def measure_ceiling(ws, torch):
    """What the machine allows a bf16 GEMM main loop, each figure sustained over about 0.4 s of back-to-back
    launches: (1) nothing but MFMAs on register operands, (2) the library's main loop alone as a square GEMM,
    (3) torch.matmul (the vendor library) on the same operands as context; each on constant operands (all ones)
    and on random ones (standard normal).  The matrix cores are power-limited and the limit depends on the data."""
    dev = torch.device("cuda:0")
    out = {"peak_tflops_nominal": BF16_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s", "measurements": []}

    def sustained(fn, flops_per_call, seconds=0.4):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        n = max(3, int(seconds * 1e3 / max(e0.elapsed_time(e1), 1e-3)))
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / n
        return round(ms, 4), round(flops_per_call / ms / 1e9, 1), n

    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    wgs, rounds = 256, 4000
    sink = torch.empty(wgs * 512, device=dev)
    for kind in ("ones", "random"):
        frag = (torch.ones(16 * 512 * 8, device=dev) if kind == "ones"
                else torch.randn(16 * 512 * 8, device=dev, generator=gen)).to(torch.bfloat16)
        ms, tf, n = sustained(lambda: ws.probe_mfma_loop(frag, rounds, wgs, sink), wgs * 8 * rounds * 128 * 16384.0)
        out["measurements"].append({"what": "MFMA only, operands in registers (256 workgroups x 8 waves)", "operands": kind,
                                    "ms_per_launch": ms, "tflops": tf, "launches": n})
    M = N = 4096
    K = 8192
    for kind in ("ones", "random"):
        mk = (lambda r, c: torch.ones((r, c), device=dev).to(torch.bfloat16)) if kind == "ones" else \
             (lambda r, c: torch.randn((r, c), device=dev, generator=gen).to(torch.bfloat16))
        A, Bm = mk(M, K), mk(N, K)
        Cm = torch.empty((N, M), device=dev, dtype=torch.bfloat16)
        ms, tf, n = sustained(lambda: ws.probe_gemm(A, Bm, Cm), 2.0 * M * N * K)
        out["measurements"].append({"what": f"library main loop alone, C = A . B^T, {M} x {N} x {K}", "operands": kind,
                                    "ms_per_launch": ms, "tflops": tf, "launches": n})
        ref = torch.matmul(Bm[:64].float(), A[:64].float().t())          # C[n][m]
        err = float((Cm[:64, :64].float() - ref).abs().max() / ref.abs().max())
        out["measurements"][-1]["max_rel_err_vs_fp32_matmul_sample"] = err
        ms, tf, n = sustained(lambda: torch.matmul(A, Bm.t(), out=Cm), 2.0 * M * N * K)
        out["measurements"].append({"what": f"torch.matmul (vendor library, context), {M} x {N} x {K}", "operands": kind,
                                    "ms_per_launch": ms, "tflops": tf, "launches": n})
    return out


def cpu_baseline(args, result, inputs, p, B, D, C, lse):
    """The oracle as it stands, on the host cores, on one full step of the same workload (or a row
    sample of it when the step would take minutes)."""
    import numpy as np
    from oracle import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    rows = B if 6.0 * B * D * C <= 2.0e12 else max(1, int(2.0e12 / (6.0 * D * C)))
    Xo = inputs.bf16_bits_to_f64(p.X_bits[:rows])
    Wo = inputs.bf16_bits_to_f64(p.W_bits)
    t0 = time.perf_counter()
    ref = oracle.unsharded(Xo, Wo, None, p.labels[:rows], 1.0)
    dt = time.perf_counter() - t0
    result["cpu_baseline"] = {
        "value": round(rows / dt, 2),
        "unit": "samples/s",
        "cores": int(cores),
        "kind": "oracle",
        "sample": f"one fwd+bwd step of the fp64 numpy oracle on {rows} of {B} rows, all {C} classes, {dt:.1f} s",
    }
    got = lse.cpu().numpy()[:rows]
    result["cpu_baseline"]["max_abs_lse_diff_vs_gpu"] = float(np.max(np.abs(got - ref["lse"])))


if __name__ == "__main__":
    main()
