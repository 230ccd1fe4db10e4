/* libwhalesplit -- the single-GPU hot path of a class-column-split fully-connected
 * layer with softmax cross-entropy, for AMD MI355X (gfx950).
 *
 * Background (Whale, arXiv 2011.09208).  The paper's motivating workload is a
 * ResNet50 feature extractor feeding a 100 000-class fully-connected layer and a
 * softmax (Section 1; Section 2.1).  Under its `split` primitive (Section 3.1.2,
 * the replicate/split listing) the FC weight is cut along the class dimension
 * (ShardingInfo [0, 1], Section 3.2.2); each device multiplies the features by its
 * own slice, and the slices' outputs concatenate to the full product (Section 2.1,
 * "Tensor Model Parallelism").  Shard widths may be uneven (Section 3.3.1).  This
 * library is what ONE device runs for its shard; several shards can be evaluated
 * one after another on the same GPU and merged with ws_combine_partials.
 *
 * Notation.  B rows (samples), D features, C_shard classes in this shard, which
 * covers global class ids [class_offset, class_offset + C_shard).
 *   z[i][c] = sum_d X[i][d] * W[c][d] + b[c]
 * Inputs are bfloat16, every accumulation is fp32.
 *
 * Memory.  EVERY pointer is a DEVICE pointer owned by the caller.  The library
 * allocates nothing, never synchronises the host, and enqueues all work on
 * `stream` (a hipStream_t passed as void*; NULL = the default stream).  Inputs are
 * never modified; outputs are fully overwritten unless stated; buffers must not
 * overlap.  Workspaces are caller-owned scratch whose contents are unspecified
 * after the call; size them with the *_workspace_bytes queries.
 *
 * Layout.  Matrices are row-major with a row pitch given in ELEMENTS.  W is stored
 * class-major, [C_shard][D] (the paper's [D, C] matrix transposed), so a column
 * shard of the layer is a contiguous slab of rows and both GEMM operands of the
 * logits product are contiguous along the contraction.
 *
 * Errors.  Every entry point returns a ws_status.  Arguments are validated on the
 * host before any HIP call, so the WS_ERR_NULL/SHAPE/ALIGN/RANGE/WORKSPACE paths
 * need no GPU.  Requirements: B, D, C_shard > 0; D a multiple of 64; every matrix (and the
 * backward call's bf16 dz scratch, 2 * roundup(B, 256) * roundup(C_shard, 256) bytes) below 4 GiB
 * with 256 rows to spare, as the kernels use 32-bit offsets (else WS_ERR_SHAPE); pitches >= D
 * (>= C for the statistics stride) and multiples of 8 elements; matrix base
 * pointers 16-byte aligned, fp32/int32 vectors 4-byte aligned;
 * class_offset >= 0 and class_offset + C_shard <= INT32_MAX.  Labels live on the
 * device and are not range-checked: a label outside the shard simply matches no
 * class of it.  A HIP launch failure is reported as WS_ERR_HIP.
 */
#ifndef WHALESPLIT_H
#define WHALESPLIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WS_OK = 0,
    WS_ERR_NULL = 1,       /* a required pointer is NULL */
    WS_ERR_SHAPE = 2,      /* non-positive size, D not a multiple of 64, pitch < row length */
    WS_ERR_ALIGN = 3,      /* pointer or pitch not aligned as required */
    WS_ERR_RANGE = 4,      /* class_offset negative or class range overflows int32; S out of range */
    WS_ERR_WORKSPACE = 5,  /* workspace NULL or smaller than the query says */
    WS_ERR_HIP = 6,        /* the HIP runtime refused a launch */
    WS_ERR_LIMIT = 7       /* ws_split_fc_fwd_static: the shape needs more than the built-in scratch */
} ws_status;

/* Human-readable name of a status code (static storage; never NULL). */
const char* ws_status_string(int status);

/* Library version, major * 1000 + minor. */
int ws_version(void);

/* Bytes of scratch ws_split_fc_fwd needs for this shape (0 on invalid shape). */
size_t ws_fwd_workspace_bytes(int32_t B, int32_t D, int32_t C_shard);

/* Forward call of one shard (Section 2.1 split matmul; Section 3.1.2 FC + Softmax
 * inside one split scope).  Computes the shard's logits tile by tile on the matrix
 * cores and reduces them in the GEMM epilogue; the [B, C_shard] logits are never
 * written to memory.  Per row i:
 *   row_max[i]     = max_c z[i][c]                       over the shard's classes
 *   row_sumexp[i]  = sum_c exp(z[i][c] - row_max[i])
 *   label_logit[i] = z[i][labels[i] - class_offset] if the label lies in the shard,
 *                    else exactly 0.0f
 * X        bf16 [B][ldx]        W_shard  bf16 [C_shard][ldw]
 * b_shard  fp32 [C_shard] or NULL (= zero bias)
 * labels   int32 [B], GLOBAL class ids
 * outputs  fp32 [B] each
 */
int ws_split_fc_fwd(const void* X, int64_t ldx,
                    const void* W_shard, int64_t ldw,
                    const float* b_shard,
                    const int32_t* labels,
                    int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                    float* row_max, float* row_sumexp, float* label_logit,
                    void* workspace, size_t workspace_bytes, void* stream);

/* The forward call for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * ws_split_fc_fwd (bit-identical outputs), but the per-class-tile partials live in a fixed array built
 * into the library's device code instead of a caller workspace; the call allocates and frees nothing.
 *   Limit: ws_fwd_workspace_bytes(B, D, C_shard) <= WS_STATIC_SCRATCH_BYTES, else WS_ERR_LIMIT (checked on
 *   the host with the other arguments, before any HIP call).  16 MiB covers one shard of every workload
 *   this library is measured on (headline 3.2 MB; B = 8192 x 50 000 classes 12.8 MB).
 *   Every GPU the library runs on holds its own 16 MiB copy of the array until the process ends.
 *   The first call on a device looks the array's device address up (hipGetSymbolAddress); make that
 *   first call outside a stream capture.
 *   All calls on one GPU share the array: two calls whose kernels may overlap on that GPU (different
 *   streams, no ordering between them) race on it.  Calls on one stream, or ordered by events, are safe;
 *   nothing in the array has to be cleared between calls. */
#define WS_STATIC_SCRATCH_BYTES (16u << 20)
int ws_split_fc_fwd_static(const void* X, int64_t ldx,
                           const void* W_shard, int64_t ldw,
                           const float* b_shard,
                           const int32_t* labels,
                           int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                           float* row_max, float* row_sumexp, float* label_logit,
                           void* stream);

/* Merge the statistics of S shards evaluated on this GPU (no collectives):
 *   m = max_s row_max[s];  sum = sum_s row_sumexp[s] * exp(row_max[s] - m)
 *   logsumexp = m + log(sum);  loss_rows = logsumexp - sum_s label_logit[s]
 * The three inputs are [S][shard_stride] fp32 arrays (row i of shard s at
 * s * shard_stride + i), shard_stride >= B, 1 <= S <= 65536.
 * loss_mean, if not NULL, receives the mean of loss_rows (one float).
 * This replaces the all-gather of logits the paper's split matmul would need
 * (Section 2.1) by an exchange of three floats per row.
 */
int ws_combine_partials(const float* row_max, const float* row_sumexp, const float* label_logit,
                        int32_t S, int32_t B, int64_t shard_stride,
                        float* logsumexp, float* loss_rows, float* loss_mean,
                        void* stream);

/* Bytes of scratch ws_split_fc_bwd needs for this shape (0 on invalid shape). */
size_t ws_bwd_workspace_bytes(int32_t B, int32_t D, int32_t C_shard);

/* Backward call of one shard, given the combined log-sum-exp of all shards.
 * Recomputes the shard's logits exactly as the forward call does, then
 *   dz[i][c]   = grad_scale * (exp(z[i][c] - logsumexp[i]) - [labels[i] == class_offset + c])
 *   dX_partial = dz . W_shard      fp32 [B][lddx]  (overwritten, or += if accumulate_dx != 0)
 *   dW_shard   = dz^T . X          bf16 [C_shard][lddw]
 *   db_shard   = column sums of dz fp32 [C_shard]   (skipped if NULL; summed before dz is rounded)
 * dz is held once, in bf16, in the workspace.  grad_scale = 1 gives the gradient of
 * the summed loss, 1/B that of the mean loss.  dX_partial is this shard's share of
 * the feature gradient: the sum over shards is the full dX (what flows back over
 * the paper's bridge layer, Section 3.2.3).  dW_shard never leaves the device that
 * owns the shard, which is the point of splitting the layer (Section 1).
 */
int ws_split_fc_bwd(const void* X, int64_t ldx,
                    const void* W_shard, int64_t ldw,
                    const float* b_shard,
                    const float* logsumexp,
                    const int32_t* labels,
                    int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                    float grad_scale,
                    float* dX_partial, int64_t lddx, int32_t accumulate_dx,
                    void* dW_shard, int64_t lddw,
                    float* db_shard,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Backward call with the weight update folded in.  A mini-batch ends with the gradients, scaled by a
 * learning rate, updating the parameters (Section 2.1); for the split classifier the gradient of a
 * shard's weights never leaves its device (Section 1), so the update can be applied where the
 * gradient is produced and dW_shard need not be written at all:
 *   W_shard[c][d] <- bf16(W_shard[c][d] - lr * dW[c][d])     in place (dW rounded to bf16 first, as
 *                                                            ws_split_fc_bwd would have stored it)
 *   b_shard[c]    <- b_shard[c] - lr * db[c]                 in place, if b_shard is not NULL
 * dX_partial is computed from the weights as they were before the call.  Everything else as in
 * ws_split_fc_bwd (same workspace size); lr must be finite (WS_ERR_RANGE).  Plain SGD only:
 * there are no optimizer states and no fp32 master copy of the weights. */
int ws_split_fc_bwd_sgd(const void* X, int64_t ldx, void* W_shard, int64_t ldw, float* b_shard,
                        const float* logsumexp, const int32_t* labels,
                        int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                        float grad_scale, float lr,
                        float* dX_partial, int64_t lddx, int32_t accumulate_dx,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Predictions of one shard.  The paper's split listing (Section 3.1.2) ends the split scope with
 * predictions = Softmax(logits); with the combined log-sum-exp of all shards every shard can write
 * its own columns of that matrix without seeing another shard's logits:
 *   P[i][c] = exp(z[i][c] - logsumexp[i])      bf16 [B][ldp], c in [0, C_shard)
 * The shards' P concatenate along the split dimension (ws_bridge_gather, dim = 1) to the full
 * softmax; each row of it sums to 1.  The logits are recomputed exactly as in the forward call
 * and are not stored.  P 16-byte aligned, ldp >= C_shard and a multiple of 8; columns beyond
 * C_shard are not touched.  No workspace. */
int ws_split_fc_predict(const void* X, int64_t ldx, const void* W_shard, int64_t ldw,
                        const float* b_shard, const float* logsumexp,
                        int32_t B, int32_t D, int32_t C_shard,
                        void* P, int64_t ldp, void* stream);

/* Arg-max predictions.  The class a row is assigned to is the arg-max of Softmax(logits), which is the
 * arg-max of the logits: every shard reports its best class and that class's logit, and the shards'
 * candidates merge by the larger logit (the partial arg-max merge that stands in for gathering the
 * split-dimension outputs, Section 3.2.3).  Among equal logits the lowest class id wins, in both calls.
 *   ws_split_fc_top1   top_logit[i] = max_c z[i][c],  top_class[i] = class_offset + argmax_c z[i][c]
 *                      (fp32 / int32 [B]); workspace of ws_fwd_workspace_bytes
 *   ws_combine_top1    top_logit / top_class [S][shard_stride] -> best_logit / best_class [B]
 * The comparison is made on the fp32 logits the kernel computes. */
int ws_split_fc_top1(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                     int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                     float* top_logit, int32_t* top_class,
                     void* workspace, size_t workspace_bytes, void* stream);
int ws_combine_top1(const float* top_logit, const int32_t* top_class, int32_t S, int32_t B,
                    int64_t shard_stride, float* best_logit, int32_t* best_class, void* stream);

/* Hardware-aware shard widths (HOST pointers only; no GPU work).  Section 3.3.1: a `split`
 * TaskGraph is balanced over devices of unequal capacity by uneven sharding in the splitting
 * dimension; load ratios proportional to the devices' FLOP/s minimise the formula given there,
 * and Algorithm 1 (Memory-Constraint Load Balancing) then shifts load from the over-memory device
 * with the highest memory utilisation to the device with room that has the lowest (FLOP
 * utilisation, memory utilisation), until no device is over memory or none has room.
 * Here the unit of load is one class column: device i with width w_i uses (w_i / C) TG_mem of
 * memory and (w_i / C) TG_flop of work.  Initial widths are the proportional shares rounded by
 * largest remainder; a shift moves the smaller of what the peak must shed and what the valley can
 * take; ties go to the lower device index.
 *   DF[N]  FLOP/s of each device        DM[N]  memory capacity of each device
 *   TG_flop, TG_mem   work and peak memory of the whole layer (same units as DF, DM)
 *   widths[N] out: non-negative, sum = C    feasible out: 1 if every device fits its memory, else 0
 * WS_ERR_NULL / WS_ERR_SHAPE (N, C <= 0) / WS_ERR_RANGE (a non-positive or non-finite quantity).
 */
int ws_balance_widths(int32_t N, const double* DF, const double* DM, double TG_flop, double TG_mem,
                      int32_t C, int32_t* widths, int32_t* feasible);

/* ---- The ends of the bridge layer on one device (Section 3.2.3) ------------------------------
 * Between two TaskGraphs with different strategies the paper inserts a bridge layer that gathers the
 * distributed outputs of the first so that the second reads a complete tensor: for `replicate` the
 * parts are different batches and are concatenated along the batch dimension, for `split` they are
 * slices along the split dimension and are concatenated there.  In the workload of this library the
 * replicated feature extractor hands its per-replica feature blocks to the split classifier
 * (gather along the batch: this builds X), and on the way back the shards' dX_partial are summed
 * and cut along the batch again.  These entry points are what ONE device runs once the parts are
 * in its memory; moving them between devices is not part of this library.
 * The part tables (arrays of pointers, pitches, extents) are HOST arrays; the pointers in them
 * are DEVICE pointers.  At most WS_BRIDGE_MAX_PARTS parts per call (else WS_ERR_RANGE). */
#define WS_BRIDGE_MAX_PARTS 64

/* Forward end: out = concatenation of n parts.
 *   dim = 0  replicate pattern: part p is [extents[p]][other], parts stack along the rows (batch)
 *   dim = 1  split pattern:     part p is [other][extents[p]], parts stack along the columns
 *   ld_parts[p], ld_out  row pitches in elements; elem_bytes 2 or 4; extents may be uneven or 0
 * Bytes are copied unchanged.  Every pointer and pitch must be a multiple of elem_bytes
 * (WS_ERR_ALIGN); wider alignment is detected and used.  out must not overlap any part. */
int ws_bridge_gather(int32_t dim, const void* const* parts, const int64_t* ld_parts,
                     const int32_t* extents, int32_t n, int32_t other, int32_t elem_bytes,
                     void* out, int64_t ld_out, void* stream);

/* Backward end in front of a split TaskGraph: the S shards each hold a partial gradient of the
 * gathered tensor (fp32 [B][ld_partials[s]], B = sum of rows[]; ws_split_fc_bwd's dX_partial);
 * replica r receives rows [rows[0] + .. + rows[r-1], +rows[r]) of their sum:
 *   out_parts[r][i][d] = sum_{s = 0 .. S-1, in this order} partials[s][row0_r + i][d]   fp32
 * D a multiple of 4; all pointers 16-byte aligned, pitches multiples of 4 and >= D. */
int ws_bridge_reduce_partition(const float* const* partials, const int64_t* ld_partials, int32_t S,
                               int32_t D, float* const* out_parts, const int64_t* ld_out,
                               const int32_t* rows, int32_t R, void* stream);

/* The fusion rule of Section 3.2.3 (HOST pointers only; no GPU work): when the bridge gathers
 * along the dimension along which the successor TaskGraph partitions its input, the gather and
 * the partition are both removed.  Reading taken here: they cancel only if the cuts coincide as
 * well (same number of parts, same extents), because otherwise data still has to change devices.
 * *fusable = 1 if both operations can be dropped, else 0. */
int ws_bridge_fusable(int32_t gather_dim, int32_t n_src, const int64_t* src_extents,
                      int32_t partition_dim, int32_t n_dst, const int64_t* dst_extents,
                      int32_t* fusable);

/* ---- The contraction-split sharding pattern, for comparison (Section 3.2.2, Section 5.3.2) --------
 * The paper's MatMul ShardingUnit has two sharding patterns: SP1 cuts the second input along its
 * second dimension (the class split every other entry point of this library implements), SP2 cuts
 * BOTH inputs along the contraction dimension and sums the full-width partial outputs with an
 * AllReduce; the paper measures SP1 1.6x to 3.75x faster.  These two calls are one device's share
 * of SP2's forward pass, kept so that the two patterns can be measured side by side:
 *   ws_sp2_partial_logits   Z_partial[i][c] = sum_{d in slice} X[i][d] * W[c][d]   fp32 [B][ldz], ALL C classes
 *   ws_sp2_reduce_stats     z = sum_s Z_partial_s (slice order s = 0 .. S-1) + bias;
 *                           logsumexp[i] = ln sum_c exp(z[i][c]);  loss_rows[i] = logsumexp[i] - z[i][labels[i]]
 * X_slice bf16 [B][ldx] and W_slice bf16 [C][ldw] hold D_slice (a multiple of 64) columns of X and
 * W; alignment and size rules as for ws_split_fc_fwd.  Z_partial (both calls): 16-byte aligned, pitch a
 * multiple of 4 elements and >= C.  Z_partials is a HOST array of S (at most 64) DEVICE pointers;
 * bias fp32 [C] 16-byte aligned or NULL. */
int ws_sp2_partial_logits(const void* X_slice, int64_t ldx, const void* W_slice, int64_t ldw,
                          int32_t B, int32_t D_slice, int32_t C,
                          float* Z_partial, int64_t ldz, void* stream);
int ws_sp2_reduce_stats(const float* const* Z_partials, const int64_t* ldz, int32_t S,
                        const float* bias, const int32_t* labels, int32_t B, int32_t C,
                        float* logsumexp, float* loss_rows, void* stream);

/* Diagnostics for benchmarks (not part of the paper's method): what the machine allows the GEMM main loop.
 * The matrix cores of this part are power-limited and the limit depends on the operand values, so the
 * caller supplies the data (e.g. all ones against random values) and times the launches itself.
 *   ws_probe_mfma_loop  `workgroups` workgroups of 8 waves; every wave runs `rounds` x 128
 *                       v_mfma_f32_16x16x32_bf16 (16384 flops each) on operands held in registers.
 *                       fragments: DEVICE, 16 x 512 x 16 bytes of bf16 values, 16-byte aligned;
 *                       sink: DEVICE fp32 [workgroups * 512] (receives a checksum so the loop is kept).
 *   ws_probe_gemm       C[n][m] = sum_k A[m][k] * B[n][k], bf16 in (A [M][lda], B [N][ldb]), bf16 out
 *                       (C [N][ldc]), fp32 accumulation: the library's shared main loop and output path
 *                       alone.  M, N multiples of 256, K of 64; 16-byte aligned, pitches multiples of 8. */
int ws_probe_mfma_loop(const void* fragments, int32_t rounds, int32_t workgroups, float* sink, void* stream);
int ws_probe_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, int32_t M, int32_t N, int32_t K,
                  void* C, int64_t ldc, void* stream);

/* Optional per-kernel timing, for benchmarks (not part of the paper's method; host-side state,
 * not thread safe).  ws_profile_enable(n) creates a pool of n event pairs (n <= 0 switches
 * timing off and frees the pool); while the pool lasts, every kernel the library launches is
 * bracketed by two events recorded on the launch stream.  ws_profile_reset() starts a new
 * measurement.  ws_profile_pause(1) lets launches go untimed until ws_profile_pause(0) (a benchmark can
 * time the kernels of every n-th step only, so that the event records perturb the step time less).
 * ws_profile_read() waits for the recorded events of one kernel (indices
 * 0 .. ws_profile_kernel_count() - 1, names from ws_profile_kernel_name) and returns the summed
 * duration in milliseconds and the number of timed launches.  total_ms and launches are HOST
 * pointers.
 *
 * ws_profile_trace_dw(trace, tiles): while `trace` (DEVICE, 8-byte aligned, uint64 [tiles][8], owned by the
 * caller, who keeps it alive until tracing is switched off and the last traced call has finished) is set,
 * the dW kernel of every backward call runs as an instrumented copy with the same arithmetic and stores;
 * for its output tile t (class tile t / (D / 256), feature tile t % (D / 256)) thread 0 of the workgroup
 * writes trace[t][0..5] = shader clock at: kernel entry, start of the main loop, end of the main loop, output
 * tile staged in LDS, row stores issued, row stores acknowledged; [6] = workgroup id; [7] = XCC_ID << 32 |
 * HW_ID (which compute unit).  A backward call with more than `tiles` output tiles returns WS_ERR_WORKSPACE
 * before launching anything.  trace = NULL switches tracing off. */
int ws_profile_enable(int32_t max_launches);
int ws_profile_reset(void);
int ws_profile_pause(int32_t paused);
int ws_profile_trace_dw(void* trace, int64_t tiles);
int32_t ws_profile_kernel_count(void);
const char* ws_profile_kernel_name(int32_t kernel);
int ws_profile_read(int32_t kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* WHALESPLIT_H */
