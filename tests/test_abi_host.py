"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ws():
    from paper_2011_09208_amd import buildlib
    if buildlib.is_stale():
        buildlib.build()
    from paper_2011_09208_amd import binding
    return binding


def test_header_symbols_are_exported(ws):
    text = open(os.path.join(ROOT, "include", "whalesplit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ws_[a-z0-9_]+)\s*\(", text))
    assert declared == set(ws.EXPORTS)
    for name in declared:
        assert getattr(ws.lib, name) is not None


def test_version_and_status_strings(ws):
    assert ws.version() >= 1000
    names = [ws.status_string(i) for i in range(8)]
    assert names == ["WS_OK", "WS_ERR_NULL", "WS_ERR_SHAPE", "WS_ERR_ALIGN", "WS_ERR_RANGE",
                     "WS_ERR_WORKSPACE", "WS_ERR_HIP", "WS_ERR_LIMIT"]
    assert ws.status_string(99) == "WS_ERR_UNKNOWN"


def test_workspace_queries(ws):
    assert ws.fwd_workspace_bytes(0, 64, 1) == 0 and ws.bwd_workspace_bytes(4, 65, 1) == 0
    # one (max, sum) pair per 256-class tile and padded row
    assert ws.fwd_workspace_bytes(1024, 2048, 100_000) == 2 * 391 * 1024 * 4
    # dz in bf16 on whole tiles (held once), X transposed, one db partial sum per 64 rows, plus the
    # split-K partial sums of dX
    b = ws.bwd_workspace_bytes(1024, 2048, 100_000)
    fixed = 1024 * 100_096 * 2 + 2048 * 1024 * 2 + 16 * 100_096 * 4
    assert b >= fixed and (b - fixed) % (1024 * 2048 * 4) == 0
    assert b < 2 * 1024 * 100_096 * 2          # no second copy of dz
    assert ws.bwd_workspace_bytes(32, 256, 500) >= 256 * 512 * 2 + 256 * 256 * 2


A = 0x10000          # fake, 16-byte aligned "device" addresses: validation never dereferences them


def _fwd(ws, X=A, ldx=64, W=A, ldw=64, b=None, y=A, B=4, D=64, C=8, off=0, m=A, s=A, t=A, wsp=A, wsb=1 << 20):
    return ws.lib.ws_split_fc_fwd(X, ldx, W, ldw, b, y, B, D, C, off, m, s, t, wsp, wsb, None)


def _bwd(ws, X=A, ldx=64, W=A, ldw=64, b=None, lse=A, y=A, B=4, D=64, C=8, off=0, g=1.0, dX=A, lddx=64,
         acc=0, dW=A, lddw=64, db=None, wsp=A, wsb=1 << 24):
    return ws.lib.ws_split_fc_bwd(X, ldx, W, ldw, b, lse, y, B, D, C, off, g, dX, lddx, acc, dW, lddw, db,
                                  wsp, wsb, None)


def test_fwd_validation(ws):
    E = {n: i for i, n in enumerate(["OK", "NULL", "SHAPE", "ALIGN", "RANGE", "WORKSPACE", "HIP"])}
    assert _fwd(ws, X=None) == E["NULL"] and _fwd(ws, W=None) == E["NULL"] and _fwd(ws, y=None) == E["NULL"]
    assert _fwd(ws, m=None) == E["NULL"] and _fwd(ws, s=None) == E["NULL"] and _fwd(ws, t=None) == E["NULL"]
    assert _fwd(ws, B=0) == E["SHAPE"] and _fwd(ws, C=-1) == E["SHAPE"] and _fwd(ws, D=72, ldx=72, ldw=72) == E["SHAPE"]
    assert _fwd(ws, ldx=32) == E["SHAPE"] and _fwd(ws, ldw=56) == E["SHAPE"]
    assert _fwd(ws, off=-1) == E["RANGE"] and _fwd(ws, off=2**31 - 4) == E["RANGE"]
    assert _fwd(ws, X=A + 2) == E["ALIGN"] and _fwd(ws, W=A + 8) == E["ALIGN"] and _fwd(ws, ldx=68) == E["ALIGN"]
    assert _fwd(ws, m=A + 2) == E["ALIGN"] and _fwd(ws, b=A + 1) == E["ALIGN"]
    assert _fwd(ws, wsp=None) == E["WORKSPACE"] and _fwd(ws, wsb=16) == E["WORKSPACE"]
    assert _fwd(ws, wsp=A + 4) == E["ALIGN"]


def test_bwd_validation(ws):
    E = {n: i for i, n in enumerate(["OK", "NULL", "SHAPE", "ALIGN", "RANGE", "WORKSPACE", "HIP"])}
    assert _bwd(ws, lse=None) == E["NULL"] and _bwd(ws, dX=None) == E["NULL"] and _bwd(ws, dW=None) == E["NULL"]
    assert _bwd(ws, X=None) == E["NULL"]
    assert _bwd(ws, D=0) == E["SHAPE"] and _bwd(ws, lddx=60) == E["SHAPE"] and _bwd(ws, lddw=8) == E["SHAPE"]
    assert _bwd(ws, off=-5) == E["RANGE"]
    assert _bwd(ws, dX=A + 4) == E["ALIGN"] and _bwd(ws, dW=A + 2) == E["ALIGN"] and _bwd(ws, lddw=68) == E["ALIGN"]
    assert _bwd(ws, db=A + 3) == E["ALIGN"] and _bwd(ws, lddx=66) == E["ALIGN"]
    assert _bwd(ws, wsb=1024) == E["WORKSPACE"] and _bwd(ws, wsp=None) == E["WORKSPACE"]


def test_combine_validation(ws):
    f = ws.lib.ws_combine_partials
    assert f(None, A, A, 1, 4, 4, A, A, None, None) == 1
    assert f(A, A, A, 1, 4, 4, None, A, None, None) == 1
    assert f(A, A, A, 1, 0, 4, A, A, None, None) == 2
    assert f(A, A, A, 2, 8, 4, A, A, None, None) == 2
    assert f(A, A, A, 0, 4, 4, A, A, None, None) == 4
    assert f(A, A, A, 70000, 4, 4, A, A, None, None) == 4
    assert f(A + 1, A, A, 1, 4, 4, A, A, None, None) == 3
    assert f(A, A, A, 1, 4, 4, A, A, A + 2, None) == 3


def test_static_forward_argument_validation(ws):
    """The entry point without a workspace validates like the forward call and refuses, on the host, a shape
    whose class-tile partials exceed the built-in scratch."""
    E = {ws.status_string(i): i for i in range(8)}

    def fwd(X=A, ldx=64, W=A, ldw=64, b=None, y=A, B=4, D=64, C=8, off=0, m=A, s=A, t=A):
        return ws.lib.ws_split_fc_fwd_static(X, ldx, W, ldw, b, y, B, D, C, off, m, s, t, None)

    assert fwd(X=None) == E["WS_ERR_NULL"] and fwd(t=None) == E["WS_ERR_NULL"]
    assert fwd(D=65) == E["WS_ERR_SHAPE"] and fwd(ldw=32) == E["WS_ERR_SHAPE"]
    assert fwd(W=A + 8) == E["WS_ERR_ALIGN"] and fwd(m=A + 2) == E["WS_ERR_ALIGN"]
    assert fwd(off=-1) == E["WS_ERR_RANGE"]
    assert ws.fwd_workspace_bytes(8192, 64, 50_000) <= ws.STATIC_SCRATCH_BYTES
    assert ws.fwd_workspace_bytes(8192, 64, 600_000) > ws.STATIC_SCRATCH_BYTES
    assert fwd(B=8192, C=600_000) == E["WS_ERR_LIMIT"]
    assert fwd(B=1 << 20, C=4096) == E["WS_ERR_LIMIT"]
    text = open(os.path.join(ROOT, "include", "whalesplit.h")).read()
    assert re.search(r"#define\s+WS_STATIC_SCRATCH_BYTES\s+\(16u\s*<<\s*20\)", text) and ws.STATIC_SCRATCH_BYTES == 16 << 20


def test_probe_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(8)}

    def gemm(A_=A, lda=64, B_=A, ldb=64, M=256, N=256, K=64, C_=A, ldc=256):
        return ws.lib.ws_probe_gemm(A_, lda, B_, ldb, M, N, K, C_, ldc, None)

    assert gemm(A_=None) == E["WS_ERR_NULL"] and gemm(C_=None) == E["WS_ERR_NULL"]
    assert gemm(M=128) == E["WS_ERR_SHAPE"] and gemm(K=32) == E["WS_ERR_SHAPE"] and gemm(ldc=128) == E["WS_ERR_SHAPE"]
    assert gemm(M=1 << 20, lda=4096, K=4096, ldc=1 << 20) == E["WS_ERR_SHAPE"]        # beyond 32-bit offsets
    assert gemm(B_=A + 8) == E["WS_ERR_ALIGN"] and gemm(lda=68) == E["WS_ERR_ALIGN"]

    def loop(frag=A, rounds=1, wgs=1, sink=A):
        return ws.lib.ws_probe_mfma_loop(frag, rounds, wgs, sink, None)

    assert loop(frag=None) == E["WS_ERR_NULL"] and loop(sink=None) == E["WS_ERR_NULL"]
    assert loop(rounds=0) == E["WS_ERR_RANGE"] and loop(wgs=0) == E["WS_ERR_RANGE"] and loop(wgs=1 << 20) == E["WS_ERR_RANGE"]
    assert loop(frag=A + 4) == E["WS_ERR_ALIGN"]


def test_predict_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(7)}

    def pred(X=A, ldx=64, W=A, ldw=64, b=None, lse=A, B=4, D=64, C=8, P=A, ldp=8):
        return ws.lib.ws_split_fc_predict(X, ldx, W, ldw, b, lse, B, D, C, P, ldp, None)

    assert pred(P=None) == E["WS_ERR_NULL"] and pred(lse=None) == E["WS_ERR_NULL"]
    assert pred(D=65) == E["WS_ERR_SHAPE"] and pred(C=0) == E["WS_ERR_SHAPE"]
    assert pred(C=9, ldp=8) == E["WS_ERR_SHAPE"]                  # pitch below the shard width
    assert pred(C=9, ldp=12) == E["WS_ERR_ALIGN"]                 # pitch not a multiple of 8
    assert pred(P=A + 2) == E["WS_ERR_ALIGN"] and pred(lse=A + 2) == E["WS_ERR_ALIGN"]
    assert pred(B=1 << 20, ldx=4096) == E["WS_ERR_SHAPE"]         # X beyond 32-bit offsets


def test_sp2_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(7)}

    def part(X=A, ldx=64, W=A, ldw=64, B=4, Ds=64, C=8, Z=A, ldz=8):
        return ws.lib.ws_sp2_partial_logits(X, ldx, W, ldw, B, Ds, C, Z, ldz, None)

    assert part(Z=None) == E["WS_ERR_NULL"]
    assert part(Ds=32) == E["WS_ERR_SHAPE"] and part(ldz=7) == E["WS_ERR_SHAPE"] and part(ldx=32) == E["WS_ERR_SHAPE"]
    assert part(X=A + 8) == E["WS_ERR_ALIGN"] and part(ldw=68) == E["WS_ERR_ALIGN"] and part(Z=A + 2) == E["WS_ERR_ALIGN"]
    # the partial-logit buffer must satisfy what the reduction requires of it later
    assert part(Z=A + 4) == E["WS_ERR_ALIGN"] and part(ldz=10) == E["WS_ERR_ALIGN"]

    def red(parts=(A, A), lds=(8, 8), S=None, bias=None, y=A, B=4, C=8, lse=A, loss=A):
        P = (ctypes.c_void_p * len(parts))(*parts)
        L = (ctypes.c_int64 * len(parts))(*lds)
        return ws.lib.ws_sp2_reduce_stats(P, L, len(parts) if S is None else S, bias, y, B, C, lse, loss, None)

    assert red(y=None) == E["WS_ERR_NULL"] and red(parts=(A, None)) == E["WS_ERR_NULL"]
    assert red(S=0) == E["WS_ERR_RANGE"] and red(parts=(A,) * 65, lds=(8,) * 65) == E["WS_ERR_RANGE"]
    assert red(C=0) == E["WS_ERR_SHAPE"] and red(lds=(8, 4)) == E["WS_ERR_SHAPE"]
    assert red(parts=(A, A + 4)) == E["WS_ERR_ALIGN"] and red(lds=(8, 10)) == E["WS_ERR_ALIGN"]
    assert red(bias=A + 4) == E["WS_ERR_ALIGN"]


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "ONE GPU" in (res.stderr + res.stdout)


def test_bwd_sgd_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(7)}

    def sgd(X=A, ldx=64, W=A, ldw=64, b=None, lse=A, y=A, B=4, D=64, C=8, off=0, g=1.0, lr=0.1, dX=A, lddx=64,
            acc=0, wsp=A, wsb=1 << 24):
        return ws.lib.ws_split_fc_bwd_sgd(X, ldx, W, ldw, b, lse, y, B, D, C, off, g, lr, dX, lddx, acc, wsp, wsb, None)

    assert sgd(W=None) == E["WS_ERR_NULL"] and sgd(dX=None) == E["WS_ERR_NULL"]
    assert sgd(lr=float("nan")) == E["WS_ERR_RANGE"] and sgd(lr=float("inf")) == E["WS_ERR_RANGE"]
    assert sgd(D=65) == E["WS_ERR_SHAPE"] and sgd(ldw=72, W=A + 8) == E["WS_ERR_ALIGN"]
    assert sgd(wsb=16) == E["WS_ERR_WORKSPACE"]


def test_top1_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(7)}

    def top(X=A, ldx=64, W=A, ldw=64, b=None, B=4, D=64, C=8, off=0, v=A, c=A, wsp=A, wsb=1 << 20):
        return ws.lib.ws_split_fc_top1(X, ldx, W, ldw, b, B, D, C, off, v, c, wsp, wsb, None)

    assert top(v=None) == E["WS_ERR_NULL"] and top(c=None) == E["WS_ERR_NULL"]
    assert top(D=96) == E["WS_ERR_SHAPE"] and top(off=-1) == E["WS_ERR_RANGE"]
    assert top(c=A + 2) == E["WS_ERR_ALIGN"] and top(wsb=8) == E["WS_ERR_WORKSPACE"]
    assert ws.lib.ws_combine_top1(A, A, 0, 4, 4, A, A, None) == E["WS_ERR_RANGE"]
    assert ws.lib.ws_combine_top1(A, A, 2, 4, 3, A, A, None) == E["WS_ERR_SHAPE"]
    assert ws.lib.ws_combine_top1(A, None, 2, 4, 4, A, A, None) == E["WS_ERR_NULL"]


def test_dw_trace_argument_validation(ws):
    E = {ws.status_string(i): i for i in range(8)}
    trace = ws.lib.ws_profile_trace_dw
    try:
        assert trace(A, 0) == E["WS_ERR_SHAPE"] and trace(A + 4, 16) == E["WS_ERR_ALIGN"]
        assert trace(A, 5) == E["WS_OK"]
        # 2 feature tiles x 3 class tiles = 6 output tiles do not fit 5 trace rows: refused before any launch
        assert _bwd(ws, D=512, ldx=512, ldw=512, lddx=512, lddw=512, C=600) == E["WS_ERR_WORKSPACE"]
        assert _bwd(ws, X=None) == E["WS_ERR_NULL"]                   # the ordinary checks still come first
    finally:
        assert trace(None, 0) == E["WS_OK"]
