"""ctypes binding over libwhalesplit.so: argument marshalling only.

Every function has the name of the C entry point it calls (minus the `ws_` prefix)
and takes torch tensors that already live on the GPU; torch is used for device
memory and the current stream, nothing else.  There is no CPU fallback: if the
library has not been built, importing this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwhalesplit.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2011_09208_amd.buildlib` "
        "(or __graft_entry__.build()); there is no fallback path")

lib = ctypes.CDLL(LIB_PATH)

_p, _i32, _i64, _sz, _f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float

lib.ws_status_string.restype = ctypes.c_char_p
lib.ws_status_string.argtypes = [ctypes.c_int]
lib.ws_version.restype = ctypes.c_int
lib.ws_version.argtypes = []
lib.ws_fwd_workspace_bytes.restype = _sz
lib.ws_fwd_workspace_bytes.argtypes = [_i32, _i32, _i32]
lib.ws_bwd_workspace_bytes.restype = _sz
lib.ws_bwd_workspace_bytes.argtypes = [_i32, _i32, _i32]
lib.ws_split_fc_fwd.restype = ctypes.c_int
lib.ws_split_fc_fwd.argtypes = [_p, _i64, _p, _i64, _p, _p, _i32, _i32, _i32, _i32, _p, _p, _p, _p, _sz, _p]
lib.ws_split_fc_fwd_static.restype = ctypes.c_int
lib.ws_split_fc_fwd_static.argtypes = [_p, _i64, _p, _i64, _p, _p, _i32, _i32, _i32, _i32, _p, _p, _p, _p]
lib.ws_combine_partials.restype = ctypes.c_int
lib.ws_combine_partials.argtypes = [_p, _p, _p, _i32, _i32, _i64, _p, _p, _p, _p]
lib.ws_split_fc_bwd.restype = ctypes.c_int
lib.ws_split_fc_bwd.argtypes = [_p, _i64, _p, _i64, _p, _p, _p, _i32, _i32, _i32, _i32, _f32,
                                _p, _i64, _i32, _p, _i64, _p, _p, _sz, _p]

lib.ws_split_fc_bwd_sgd.restype = ctypes.c_int
lib.ws_split_fc_bwd_sgd.argtypes = [_p, _i64, _p, _i64, _p, _p, _p, _i32, _i32, _i32, _i32, _f32, _f32,
                                    _p, _i64, _i32, _p, _sz, _p]
lib.ws_split_fc_top1.restype = ctypes.c_int
lib.ws_split_fc_top1.argtypes = [_p, _i64, _p, _i64, _p, _i32, _i32, _i32, _i32, _p, _p, _p, _sz, _p]
lib.ws_combine_top1.restype = ctypes.c_int
lib.ws_combine_top1.argtypes = [_p, _p, _i32, _i32, _i64, _p, _p, _p]
lib.ws_split_fc_predict.restype = ctypes.c_int
lib.ws_split_fc_predict.argtypes = [_p, _i64, _p, _i64, _p, _p, _i32, _i32, _i32, _p, _i64, _p]

lib.ws_probe_mfma_loop.restype = ctypes.c_int
lib.ws_probe_mfma_loop.argtypes = [_p, _i32, _i32, _p, _p]
lib.ws_probe_gemm.restype = ctypes.c_int
lib.ws_probe_gemm.argtypes = [_p, _i64, _p, _i64, _i32, _i32, _i32, _p, _i64, _p]

lib.ws_profile_enable.restype = ctypes.c_int
lib.ws_profile_enable.argtypes = [_i32]
lib.ws_profile_reset.restype = ctypes.c_int
lib.ws_profile_reset.argtypes = []
lib.ws_profile_pause.restype = ctypes.c_int
lib.ws_profile_pause.argtypes = [_i32]
lib.ws_profile_trace_dw.restype = ctypes.c_int
lib.ws_profile_trace_dw.argtypes = [ctypes.c_void_p, _i64]
lib.ws_profile_kernel_count.restype = _i32
lib.ws_profile_kernel_count.argtypes = []
lib.ws_profile_kernel_name.restype = ctypes.c_char_p
lib.ws_profile_kernel_name.argtypes = [_i32]
lib.ws_profile_read.restype = ctypes.c_int
lib.ws_profile_read.argtypes = [_i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]

lib.ws_balance_widths.restype = ctypes.c_int
lib.ws_balance_widths.argtypes = [_i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                  ctypes.c_double, ctypes.c_double, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]

lib.ws_bridge_gather.restype = ctypes.c_int
lib.ws_bridge_gather.argtypes = [_i32, ctypes.POINTER(_p), ctypes.POINTER(_i64), ctypes.POINTER(_i32), _i32, _i32, _i32,
                                 _p, _i64, _p]
lib.ws_bridge_reduce_partition.restype = ctypes.c_int
lib.ws_bridge_reduce_partition.argtypes = [ctypes.POINTER(_p), ctypes.POINTER(_i64), _i32, _i32, ctypes.POINTER(_p),
                                           ctypes.POINTER(_i64), ctypes.POINTER(_i32), _i32, _p]
lib.ws_bridge_fusable.restype = ctypes.c_int
lib.ws_bridge_fusable.argtypes = [_i32, _i32, ctypes.POINTER(_i64), _i32, _i32, ctypes.POINTER(_i64), ctypes.POINTER(_i32)]

lib.ws_sp2_partial_logits.restype = ctypes.c_int
lib.ws_sp2_partial_logits.argtypes = [_p, _i64, _p, _i64, _i32, _i32, _i32, _p, _i64, _p]
lib.ws_sp2_reduce_stats.restype = ctypes.c_int
lib.ws_sp2_reduce_stats.argtypes = [ctypes.POINTER(_p), ctypes.POINTER(_i64), _i32, _p, _p, _i32, _i32, _p, _p, _p]

STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = ["ws_status_string", "ws_version", "ws_fwd_workspace_bytes", "ws_split_fc_fwd", "ws_split_fc_fwd_static",
           "ws_combine_partials", "ws_bwd_workspace_bytes", "ws_split_fc_bwd", "ws_split_fc_bwd_sgd", "ws_split_fc_predict", "ws_split_fc_top1", "ws_combine_top1",
           "ws_profile_enable", "ws_profile_reset", "ws_profile_pause", "ws_profile_trace_dw", "ws_profile_kernel_count", "ws_profile_kernel_name",
           "ws_profile_read", "ws_balance_widths",
           "ws_bridge_gather", "ws_bridge_reduce_partition", "ws_bridge_fusable",
           "ws_sp2_partial_logits", "ws_sp2_reduce_stats", "ws_probe_mfma_loop", "ws_probe_gemm"]


class WhaleSplitError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__(lib.ws_status_string(self.status).decode())


def _check(status):
    if status != 0:
        raise WhaleSplitError(status)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def status_string(status):
    return lib.ws_status_string(int(status)).decode()


def version():
    return lib.ws_version()


def fwd_workspace_bytes(B, D, C_shard):
    return lib.ws_fwd_workspace_bytes(B, D, C_shard)


def bwd_workspace_bytes(B, D, C_shard):
    return lib.ws_bwd_workspace_bytes(B, D, C_shard)


def split_fc_fwd(X, W_shard, b_shard, labels, class_offset, row_max, row_sumexp, label_logit, workspace):
    """X bf16 [B, D]; W_shard bf16 [C_shard, D]; b_shard fp32 [C_shard] or None; labels int32 [B];
    outputs fp32 [B]; workspace uint8 of at least fwd_workspace_bytes."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_fwd(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard),
                               _ptr(labels), B, D, C, int(class_offset), _ptr(row_max), _ptr(row_sumexp),
                               _ptr(label_logit), _ptr(workspace), workspace.numel() * workspace.element_size(),
                               _stream()))


def split_fc_fwd_static(X, W_shard, b_shard, labels, class_offset, row_max, row_sumexp, label_logit):
    """split_fc_fwd without a workspace: the library's built-in device scratch is used (no allocation)."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_fwd_static(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard),
                                      _ptr(labels), B, D, C, int(class_offset), _ptr(row_max), _ptr(row_sumexp),
                                      _ptr(label_logit), _stream()))


def combine_partials(row_max, row_sumexp, label_logit, logsumexp, loss_rows, loss_mean=None):
    """Statistics are fp32 [S, B] (row pitch = stride(0)); outputs fp32 [B]; loss_mean fp32 [1] or None."""
    S, B = row_max.shape
    stride = row_max.stride(0) if S > 1 else max(B, row_max.stride(0))
    assert row_sumexp.shape == row_max.shape and label_logit.shape == row_max.shape
    if S > 1:
        assert row_sumexp.stride(0) == stride and label_logit.stride(0) == stride
    _check(lib.ws_combine_partials(_ptr(row_max), _ptr(row_sumexp), _ptr(label_logit), S, B, stride,
                                   _ptr(logsumexp), _ptr(loss_rows), _ptr(loss_mean), _stream()))


def split_fc_bwd(X, W_shard, b_shard, logsumexp, labels, class_offset, grad_scale, dX_partial, accumulate_dx,
                 dW_shard, db_shard, workspace):
    """dX_partial fp32 [B, D]; dW_shard bf16 [C_shard, D]; db_shard fp32 [C_shard] or None."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_bwd(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard),
                               _ptr(logsumexp), _ptr(labels), B, D, C, int(class_offset), float(grad_scale),
                               _ptr(dX_partial), dX_partial.stride(0), int(bool(accumulate_dx)),
                               _ptr(dW_shard), dW_shard.stride(0), _ptr(db_shard), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream()))


def split_fc_bwd_sgd(X, W_shard, b_shard, logsumexp, labels, class_offset, grad_scale, lr, dX_partial,
                     accumulate_dx, workspace):
    """As split_fc_bwd, but W_shard (bf16) and b_shard (fp32 or None) are updated in place by -lr * gradient."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_bwd_sgd(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard),
                                   _ptr(logsumexp), _ptr(labels), B, D, C, int(class_offset), float(grad_scale),
                                   float(lr), _ptr(dX_partial), dX_partial.stride(0), int(bool(accumulate_dx)),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def split_fc_top1(X, W_shard, b_shard, class_offset, top_logit, top_class, workspace):
    """top_logit fp32 [B], top_class int32 [B] <- the shard's best class per row."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_top1(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard), B, D, C,
                                int(class_offset), _ptr(top_logit), _ptr(top_class), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream()))


def combine_top1(top_logit, top_class, best_logit, best_class):
    """[S, B] candidates -> [B] winners."""
    S, B = top_logit.shape
    stride = top_logit.stride(0) if S > 1 else max(B, top_logit.stride(0))
    assert top_class.shape == top_logit.shape and (S == 1 or top_class.stride(0) == stride)
    _check(lib.ws_combine_top1(_ptr(top_logit), _ptr(top_class), S, B, stride, _ptr(best_logit), _ptr(best_class),
                               _stream()))


def split_fc_predict(X, W_shard, b_shard, logsumexp, P):
    """P bf16 [B, C_shard] (row pitch a multiple of 8) <- exp(z - logsumexp)."""
    B, D = X.shape
    C = W_shard.shape[0]
    _check(lib.ws_split_fc_predict(_ptr(X), X.stride(0), _ptr(W_shard), W_shard.stride(0), _ptr(b_shard),
                                   _ptr(logsumexp), B, D, C, _ptr(P), P.stride(0), _stream()))


def profile_enable(max_launches):
    _check(lib.ws_profile_enable(int(max_launches)))


def profile_reset():
    _check(lib.ws_profile_reset())


def profile_pause(paused):
    _check(lib.ws_profile_pause(int(bool(paused))))


def profile_trace_dw(trace):
    """trace: int64 CUDA tensor [tiles, 8] that the dW kernel of the following backward calls fills with
    per-tile clock stamps (see the header), or None to switch tracing off."""
    if trace is None:
        _check(lib.ws_profile_trace_dw(None, 0))
    else:
        assert trace.dtype == torch.int64 and trace.is_contiguous() and trace.shape[1] == 8
        _check(lib.ws_profile_trace_dw(_ptr(trace), trace.shape[0]))


def profile_read():
    """{kernel name: (total_ms, launches)} for every kernel that was timed since the last reset."""
    out = {}
    for k in range(lib.ws_profile_kernel_count()):
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(lib.ws_profile_read(k, ctypes.byref(ms), ctypes.byref(n)))
        if n.value:
            out[lib.ws_profile_kernel_name(k).decode()] = (ms.value, n.value)
    return out


def balance_widths(C, DF, DM, TG_flop, TG_mem):
    """Shard widths for devices with FLOP/s DF and memory DM; returns (list of widths, feasible)."""
    n = len(DF)
    df = (ctypes.c_double * n)(*[float(v) for v in DF])
    dm = (ctypes.c_double * n)(*[float(v) for v in DM])
    w = (_i32 * n)()
    ok = _i32(0)
    _check(lib.ws_balance_widths(n, df, dm, float(TG_flop), float(TG_mem), int(C), w, ctypes.byref(ok)))
    return list(w), bool(ok.value)


def bridge_gather_args(dim, parts, out):
    """The argument tuple of ws_bridge_gather (without the stream) for 2-D device tensors."""
    n = len(parts)
    other = out.shape[1 - dim]
    for p in parts:
        assert p.dtype == out.dtype and p.dim() == 2 and p.shape[1 - dim] == other
        assert p.shape[1] <= 1 or p.stride(1) == 1
    ptrs = (_p * n)(*[p.data_ptr() for p in parts])
    lds = (_i64 * n)(*[p.stride(0) if p.shape[0] > 1 else max(p.shape[1], p.stride(0)) for p in parts])
    ext = (_i32 * n)(*[p.shape[dim] for p in parts])
    return (int(dim), ptrs, lds, ext, n, int(other), out.element_size(), _ptr(out), out.stride(0))


def bridge_gather(dim, parts, out):
    """Concatenates 2-D device tensors `parts` (same dtype, 2 or 4 bytes per element) into `out` along
    dim 0 (rows: the replicate pattern) or dim 1 (columns: the split pattern)."""
    _check(lib.ws_bridge_gather(*bridge_gather_args(dim, parts, out), _stream()))


def bridge_reduce_partition_args(partials, out_parts):
    """The argument tuple of ws_bridge_reduce_partition (without the stream)."""
    S, R = len(partials), len(out_parts)
    D = partials[0].shape[1]
    assert sum(o.shape[0] for o in out_parts) <= min(p.shape[0] for p in partials)
    pp = (_p * S)(*[p.data_ptr() for p in partials])
    pl = (_i64 * S)(*[p.stride(0) for p in partials])
    op = (_p * R)(*[o.data_ptr() for o in out_parts])
    ol = (_i64 * R)(*[o.stride(0) if o.shape[0] > 1 else max(D, o.stride(0)) for o in out_parts])
    rows = (_i32 * R)(*[o.shape[0] for o in out_parts])
    return (pp, pl, S, int(D), op, ol, rows, R)


def bridge_reduce_partition(partials, out_parts):
    """out_parts[r] (fp32 [rows_r, D]) = rows of sum(partials) (fp32 [B, D] each), B = sum of rows_r."""
    _check(lib.ws_bridge_reduce_partition(*bridge_reduce_partition_args(partials, out_parts), _stream()))


def bridge_fusable(gather_dim, src_extents, partition_dim, dst_extents):
    a = (_i64 * len(src_extents))(*[int(v) for v in src_extents])
    b = (_i64 * len(dst_extents))(*[int(v) for v in dst_extents])
    ok = _i32(0)
    _check(lib.ws_bridge_fusable(int(gather_dim), len(src_extents), a, int(partition_dim), len(dst_extents), b,
                                 ctypes.byref(ok)))
    return bool(ok.value)


def sp2_partial_logits(X_slice, W_slice, Z_partial):
    """Z_partial fp32 [B, C] <- X_slice [B, D_s] . W_slice [C, D_s]^T (column slices may be views)."""
    B, Ds = X_slice.shape
    C = W_slice.shape[0]
    _check(lib.ws_sp2_partial_logits(_ptr(X_slice), X_slice.stride(0), _ptr(W_slice), W_slice.stride(0), B, Ds, C,
                                     _ptr(Z_partial), Z_partial.stride(0), _stream()))


def sp2_reduce_stats(Z_partials, bias, labels, logsumexp, loss_rows):
    S = len(Z_partials)
    B, C = Z_partials[0].shape
    zp = (_p * S)(*[z.data_ptr() for z in Z_partials])
    zl = (_i64 * S)(*[z.stride(0) for z in Z_partials])
    _check(lib.ws_sp2_reduce_stats(zp, zl, S, _ptr(bias), _ptr(labels), B, C, _ptr(logsumexp), _ptr(loss_rows),
                                   _stream()))


def probe_mfma_loop(fragments, rounds, workgroups, sink):
    """fragments: uint8/bf16 tensor of 16 * 512 * 16 bytes; sink fp32 [workgroups * 512]."""
    _check(lib.ws_probe_mfma_loop(_ptr(fragments), int(rounds), int(workgroups), _ptr(sink), _stream()))


def probe_gemm(A, B, C):
    """C [N, M] bf16 <- A [M, K] . B [N, K]^T (bf16), the library's main loop alone."""
    M, K = A.shape
    N = B.shape[0]
    _check(lib.ws_probe_gemm(_ptr(A), A.stride(0), _ptr(B), B.stride(0), M, N, K, _ptr(C), C.stride(0), _stream()))
