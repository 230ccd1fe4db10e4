// libwhalesplit: kernels and C-ABI entry points (see include/whalesplit.h for the contract).
//
// Kernels, in the order one training step of a shard runs them:
//   fwd_logits_stats   z^T tile = W_s . X^T on the matrix cores; per-row max / sum-exp / label
//                      logit reduced in the epilogue; one (max, sum) partial per 256-class tile
//   merge_class_tiles  merges those partials into row_max / row_sumexp of the shard
//   combine_partials   merges the shards' statistics into logsumexp and loss
//   bwd_recompute_dz   same GEMM again, epilogue dz = g (exp(z - lse) - onehot) stored as bf16
//                      [row][class]; column sums of the tile (db partials); its surplus workgroups
//                      write X^T for the dW contraction
//   predict_probs      softmax probabilities of the shard's classes, exp(z - lse), bf16
//   top1_logits        the shard's arg-max class and its logit per row (+ merge_top1, also used across shards)
//   bwd_dx             dX_partial = dz . W_s, split along the class contraction; partial sums
//   bwd_dw             dW_s = dz^T . X; its surplus workgroups sum the split-K partials of dX
//                      (optionally accumulating into the caller's dX) and the db partials
// fwd_logits_stats and bwd_recompute_dz run the tiles of a ragged last round (256 compute units) as
// four thin 256 x 64 tiles each (logits_thin, fwd_stats_thin, dz_thin; plan_tiles on the host); bwd_dw
// does the same where the contraction is long (dw_thin).
// Tile orders and cache reuse: each XCD walks a contiguous range of tiles whose neighbours share operand
// panels (logits_tile_coords, bwd_dx, dw_tile); every other round of tiles walks the contraction backwards
// (logits_descending, dw_tile) and bwd_recompute_dz starts with the tiles that fwd_logits_stats ended on.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <limits.h>
#include <math.h>
#include <stdint.h>

#include "../../include/whalesplit.h"
#include "gemm_core.h"

namespace ws {

constexpr float NEG_INF = -INFINITY;
constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float lane_xor(float v, int mask) { return __shfl_xor(v, mask, 64); }

// Merge of two (max, sum-exp) pairs; either may be the empty pair (-inf, 0).
__device__ __forceinline__ void merge_ms(float& m, float& s, float m2, float s2) {
    const float M = fmaxf(m, m2);
    const float f1 = (m == NEG_INF) ? 0.0f : __expf(m - M);
    const float f2 = (m2 == NEG_INF) ? 0.0f : __expf(m2 - M);
    s = s * f1 + s2 * f2;
    m = M;
}

// Class id (relative to the wave's first class) held in accumulator register v of M-tile mt by the
// lanes of 16-lane group g.
__device__ __forceinline__ int acc_row(int mt, int v, int g) { return 16 * mt + 4 * g + v; }

// z = acc + bias, with classes beyond the shard set to -inf.  `c_rel0` = the wave's first class
// relative to the workgroup's tile, `c_left` = number of valid classes from the wave's first class.
__device__ __forceinline__ void add_bias_and_mask(acc_t& acc, const float* sbias, bool has_bias, int c_rel0,
                                                  int c_left, int g) {
    if (has_bias) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 b4 = *reinterpret_cast<const f32x4*>(sbias + c_rel0 + 16 * mt + 4 * g);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] += b4;
        }
    }
    if (c_left < WAVE_M) {   // wave-uniform: only the ragged last class tile pays for masking
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (acc_row(mt, v, g) >= c_left) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[mt][nt][v] = NEG_INF;
                }
    }
}

struct FcArgs {
    const uint16_t* X; int64_t ldx;
    const uint16_t* W; int64_t ldw;
    const float* bias;
    const int32_t* labels;
    int B, D, C, class_offset;
    int Bpad;        // B rounded up to 256
    int nBT, nCT;    // tiles along the batch and class dimensions
    TilePlan plan;   // which of the nBT * nCT tiles run as full tiles and which as four thin tiles each
    int last_tile_first;   // walk the full tiles from the last to the first
};

// The tile a workgroup of a logits kernel works on: full (piece < 0) or thin piece 0 .. 3 of it.
struct TileRef {
    int ct, bt, piece;
    bool valid;
};

// Tile t of a logits launch -> (class tile, batch tile).  Up to four batch tiles: batch tiles fastest, so the 32
// consecutive tiles that an XCD runs at a time share a W panel four ways and cover 32 / nBT class tiles.  More
// batch tiles: blocks of 8 class tiles x 4 batch tiles (12 operand panels for 32 tiles instead of 33), the
// batch blocks of one block of class tiles one after the other, so that consecutive rounds share its W panels.
__device__ __forceinline__ void logits_tile_coords(const FcArgs& a, int t, int& ct, int& bt) {
    if (a.nBT <= 4) {
        ct = t / a.nBT;
        bt = t % a.nBT;
        return;
    }
    const int per_block = 8 * a.nBT;
    const int cb = t / per_block, r = t - cb * per_block;
    const int rest = a.nCT - 8 * cb, h = rest < 8 ? rest : 8;     // class tiles in this block
    const int full_bb = a.nBT >> 2, in_full = h * 4 * full_bb;
    if (r < in_full) {
        const int bb = r / (h * 4), q = r - bb * (h * 4);
        ct = 8 * cb + (q >> 2);
        bt = 4 * bb + (q & 3);
    } else {
        const int w = a.nBT & 3, q = r - in_full;
        ct = 8 * cb + q / w;
        bt = 4 * full_bb + q % w;
    }
}

__device__ __forceinline__ TileRef logits_tile_ref(const FcArgs& a) {
    TileRef r;
    r.piece = -1;
    int tile;
    if ((int)blockIdx.x >= a.plan.thin_first) {
        const int q = (int)blockIdx.x - a.plan.thin_first;
        tile = q < a.plan.n_thin ? a.plan.n_full + (q >> 2) : -1;
        r.piece = q & 3;
    } else {
        tile = xcd_logical_tile(a.plan.n_full);
        if (a.last_tile_first && tile >= 0) tile = a.plan.n_full - 1 - tile;
    }
    r.valid = tile >= 0;
    r.ct = r.bt = 0;
    if (r.valid) logits_tile_coords(a, tile, r.ct, r.bt);
    return r;
}

// Direction in which the logits of tile (ct, bt) walk the features.  A compute unit's next tile lies about 32
// tile ids further on, in the next group of class tiles (up to four batch tiles) or the next batch block of the
// same class tiles (more); alternating the direction between such groups lets it find the end of the panels
// that the two tiles share, which it has just read, still in the L2 (launches of one round have nothing to gain
// and keep one direction).  A function of the tile's coordinates and the launch shape alone, so that every
// kernel (and the thin and the full version of a tile) adds the products of a logit in the same order.
__device__ __forceinline__ bool logits_descending(const FcArgs& a, int ct, int bt) {
    if (a.nBT * a.nCT <= 256) return false;
    if (a.nBT <= 4) return (((ct * a.nBT) >> 5) & 1) != 0;
    return (((ct >> 3) ^ (bt >> 2)) & 1) != 0;
}

// Runs the logits GEMM of one 256-class x 256-row tile and leaves z (bias added, padding = -inf)
// in acc.  M = classes (A = W_s, KC), N = batch rows (B operand = X, KC), K = D.
__device__ __forceinline__ void logits_tile(acc_t& acc, const FcArgs& a, int ct, int bt, char* lds,
                                            float* sbias) {
    zero_acc(acc);
    const Operand A = make_operand(a.W, a.ldw, a.C, a.D);
    const Operand Bo = make_operand(a.X, a.ldx, a.B, a.D);
    gemm_mainloop<KC, KC>(acc, A, Bo, ct * TILE_M, bt * TILE_N, 0, a.D / TILE_K, lds, logits_descending(a, ct, bt));
    const int tid = threadIdx.x;
    const bool has_bias = a.bias != nullptr;
    if (has_bias) {
        if (tid < TILE_M) {
            const int c = ct * TILE_M + tid;
            sbias[tid] = c < a.C ? a.bias[c] : 0.0f;
        }
        __syncthreads();
    }
    const int wm = (tid >> 6) >> 2;
    add_bias_and_mask(acc, sbias, has_bias, wm * WAVE_M, a.C - (ct * TILE_M + wm * WAVE_M), (tid & 63) >> 4);
}

// Class id (relative to the wave's first class) of accumulator register v of M-tile mt in a thin tile
// is the same expression, with two M-tiles per wave instead of eight.
//
// z of thin tile `piece` (rows 64 * piece .. + 63 of batch tile bt), bias added, padding = -inf.
__device__ __forceinline__ void logits_thin(thin_acc_t& acc, const FcArgs& a, int ct, int bt, int piece, char* lds,
                                            float* sbias) {
#pragma unroll
    for (int i = 0; i < THIN_MT; ++i)
#pragma unroll
        for (int j = 0; j < THIN_NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const Operand A = make_operand(a.W, a.ldw, a.C, a.D);
    const Operand Bo = make_operand(a.X, a.ldx, a.B, a.D);
    thin_mainloop(acc, A, Bo, ct * TILE_M, bt * TILE_N + piece * THIN_N, 0, a.D / TILE_K, lds, logits_descending(a, ct, bt));
    const int tid = threadIdx.x, wave = tid >> 6, g = (tid & 63) >> 4;
    if (a.bias != nullptr) {
        if (tid < TILE_M) {
            const int c = ct * TILE_M + tid;
            sbias[tid] = c < a.C ? a.bias[c] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt) {
            const f32x4 b4 = *reinterpret_cast<const f32x4*>(sbias + wave * THIN_WAVE_M + 16 * mt + 4 * g);
#pragma unroll
            for (int nt = 0; nt < THIN_NT; ++nt) acc[mt][nt] += b4;
        }
    }
    const int c_left = a.C - (ct * TILE_M + wave * THIN_WAVE_M);
    if (c_left < THIN_WAVE_M) {
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (acc_row(mt, v, g) >= c_left) {
#pragma unroll
                    for (int nt = 0; nt < THIN_NT; ++nt) acc[mt][nt][v] = NEG_INF;
                }
    }
}

// Forward statistics of a thin tile: every wave reduces its 32 classes per row, the eight waves'
// pairs are merged through LDS in wave order.
__device__ __forceinline__ void fwd_stats_thin(const FcArgs& a, const TileRef& r, char* lds,
                                               float* __restrict__ part_max, float* __restrict__ part_sum,
                                               float* __restrict__ label_logit) {
    float* sbias = reinterpret_cast<float*>(lds);
    float* red_m = sbias + 256;            // [8][64]
    float* red_s = red_m + 512;
    thin_acc_t acc;
    logits_thin(acc, a, r.ct, r.bt, r.piece, lds, sbias);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, jl = lane & 15;
    const int cw0 = r.ct * TILE_M + wave * THIN_WAVE_M;
    const int row0 = r.bt * TILE_N + r.piece * THIN_N;
#pragma unroll
    for (int nt = 0; nt < THIN_NT; ++nt) {
        const int row = row0 + 16 * nt + jl;
        float mx = NEG_INF;
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) mx = fmaxf(mx, acc[mt][nt][v]);
        const float ms = (mx == NEG_INF) ? 0.0f : mx;
        const float shift = -ms * LOG2E;
        float s = 0.0f;
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) s += __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][v], LOG2E, shift));
        merge_ms(mx, s, lane_xor(mx, 16), lane_xor(s, 16));
        merge_ms(mx, s, lane_xor(mx, 32), lane_xor(s, 32));
        if (g == 0) {
            red_m[wave * THIN_N + 16 * nt + jl] = mx;
            red_s[wave * THIN_N + 16 * nt + jl] = s;
        }
        const bool row_ok = row < a.B;
        const int local = row_ok ? a.labels[row] - a.class_offset : -1;
        const bool in_shard = local >= 0 && local < a.C;
        const int rel = local - cw0;
        const bool mine = in_shard && rel >= 0 && rel < THIN_WAVE_M && ((rel & 15) >> 2) == g;
        if (__any(mine)) {
            float t = 0.0f;
#pragma unroll
            for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (acc_row(mt, v, g) == rel) t = acc[mt][nt][v];
            if (mine) label_logit[row] = t;
        }
        if (r.ct == 0 && wave == 0 && g == 0 && row_ok && !in_shard) label_logit[row] = 0.0f;
    }
    __syncthreads();
    if (tid < THIN_N) {
        float m = red_m[tid], s = red_s[tid];
#pragma unroll
        for (int w = 1; w < 8; ++w) merge_ms(m, s, red_m[w * THIN_N + tid], red_s[w * THIN_N + tid]);
        const int64_t o = (int64_t)r.ct * a.Bpad + row0 + tid;
        part_max[o] = m;
        part_sum[o] = s;
    }
}

__global__ __launch_bounds__(NTHREADS) void fwd_logits_stats(FcArgs a, float* __restrict__ part_max,
                                                              float* __restrict__ part_sum,
                                                              float* __restrict__ label_logit) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    float* sbias = reinterpret_cast<float*>(lds);          // reused after the main loop
    float* red_m = reinterpret_cast<float*>(lds) + 256;    // [2][256]
    float* red_s = red_m + 512;
    const TileRef ref = logits_tile_ref(a);
    if (!ref.valid) return;
    if (ref.piece >= 0) {
        fwd_stats_thin(a, ref, lds, part_max, part_sum, label_logit);
        return;
    }
    const int ct = ref.ct, bt = ref.bt;

    acc_t acc;
    logits_tile(acc, a, ct, bt, lds, sbias);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
    const int cw0 = ct * TILE_M + wm * WAVE_M;           // first class of this wave (shard-local)

    // A lane holds, for each of its four rows (one per N tile), 32 of the wave's 128 classes; the other
    // three 16-lane groups hold the rest.
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = bt * TILE_N + wn * WAVE_N + 16 * nt + jl;
        float mx = NEG_INF;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) mx = fmaxf(mx, acc[mt][nt][v]);
        const float ms = (mx == NEG_INF) ? 0.0f : mx;
        const float shift = -ms * LOG2E;                 // exp(z - m) = exp2(z * log2 e - m * log2 e)
        float s = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) s += __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][v], LOG2E, shift));
        merge_ms(mx, s, lane_xor(mx, 16), lane_xor(s, 16));
        merge_ms(mx, s, lane_xor(mx, 32), lane_xor(s, 32));
        if (g == 0) {
            red_m[wm * 256 + wn * WAVE_N + 16 * nt + jl] = mx;
            red_s[wm * 256 + wn * WAVE_N + 16 * nt + jl] = s;
        }

        // Label logit.  Exactly one lane of the whole grid holds z[row][label - offset] when the label
        // lies in the shard; rows whose label lies outside get 0 from the first class tile.
        const bool row_ok = row < a.B;
        const int local = row_ok ? a.labels[row] - a.class_offset : -1;
        const bool in_shard = local >= 0 && local < a.C;
        const int rel = local - cw0;
        const bool mine = in_shard && rel >= 0 && rel < WAVE_M && ((rel & 15) >> 2) == g;
        if (__any(mine)) {
            float t = 0.0f;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (acc_row(mt, v, g) == rel) t = acc[mt][nt][v];
            if (mine) label_logit[row] = t;
        }
        if (ct == 0 && wm == 0 && g == 0 && row_ok && !in_shard) label_logit[row] = 0.0f;
    }
    __syncthreads();
    if (tid < 256) {
        float m = red_m[tid], s = red_s[tid];
        merge_ms(m, s, red_m[256 + tid], red_s[256 + tid]);
        const int64_t o = (int64_t)ct * a.Bpad + bt * TILE_N + tid;
        part_max[o] = m;
        part_sum[o] = s;
    }
}

// One workgroup merges the class-tile partials of 16 rows: thread (r, q) folds tiles q, q + 64, ...
// of row r online, then the 64 partial pairs of a row are merged through LDS in a fixed order
// (8 groups of 8, then the 8 group results).
__global__ __launch_bounds__(1024) void merge_class_tiles(const float* __restrict__ part_max,
                                                           const float* __restrict__ part_sum, int nCT, int Bpad,
                                                           int B, float* __restrict__ row_max,
                                                           float* __restrict__ row_sumexp) {
    __shared__ float sm[64][16], ss[64][16];
    const int r = threadIdx.x & 15, q = threadIdx.x >> 4;
    const int i = blockIdx.x * 16 + r;          // < Bpad: the partial arrays are padded to whole tiles
    float m = NEG_INF, s = 0.0f;
    for (int t = q; t < nCT; t += 64) merge_ms(m, s, part_max[(int64_t)t * Bpad + i], part_sum[(int64_t)t * Bpad + i]);
    sm[q][r] = m;
    ss[q][r] = s;
    __syncthreads();
    if (q < 8) {
        m = sm[8 * q][r];
        s = ss[8 * q][r];
#pragma unroll
        for (int k = 1; k < 8; ++k) merge_ms(m, s, sm[8 * q + k][r], ss[8 * q + k][r]);
    }
    __syncthreads();
    if (q < 8) {
        sm[q][r] = m;
        ss[q][r] = s;
    }
    __syncthreads();
    if (q == 0 && i < B) {
#pragma unroll
        for (int k = 1; k < 8; ++k) merge_ms(m, s, sm[k][r], ss[k][r]);
        row_max[i] = m;
        row_sumexp[i] = s;
    }
}

__global__ void combine_partials_kernel(const float* __restrict__ row_max, const float* __restrict__ row_sumexp,
                                        const float* __restrict__ label_logit, int S, int B, int64_t stride,
                                        float* __restrict__ logsumexp, float* __restrict__ loss_rows) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    float m = NEG_INF;
    for (int s = 0; s < S; ++s) m = fmaxf(m, row_max[s * stride + i]);
    float tot = 0.0f, t = 0.0f;
    for (int s = 0; s < S; ++s) {
        const float ms = row_max[s * stride + i];
        if (ms != NEG_INF) tot += row_sumexp[s * stride + i] * __expf(ms - m);
        t += label_logit[s * stride + i];
    }
    const float lse = m + __logf(tot);
    logsumexp[i] = lse;
    loss_rows[i] = lse - t;
}

// Mean of loss_rows in a fixed summation order (one workgroup).
__global__ __launch_bounds__(1024) void mean_loss_kernel(const float* __restrict__ loss_rows, int B,
                                                          float* __restrict__ loss_mean) {
    __shared__ float red[1024];
    float acc = 0.0f;
    for (int i = threadIdx.x; i < B; i += 1024) acc += loss_rows[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss_mean = red[0] / (float)B;
}

// XT[d][b] = X[b][d], zero for b >= B (the dW contraction reads whole 64-row k-steps), in 64 x 64
// tiles through LDS.  Run by the workgroups of bwd_recompute_dz beyond its GEMM tiles: they are handed
// out last, onto compute units the final, partial round of GEMM tiles leaves idle.
struct XtArgs {
    uint16_t* XT; int64_t ldxt;          // [D][Bpad]
    int first_block, n_blocks;           // workgroups [first_block, first_block + n_blocks) transpose
};

__device__ __forceinline__ void transpose_x_tiles(const FcArgs& a, const XtArgs& x, int worker, char* lds) {
    uint16_t (*tile)[66] = reinterpret_cast<uint16_t (*)[66]>(lds);
    const int nb = a.Bpad / 64, n_tiles = nb * (a.D / 64);
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int t = worker; t < n_tiles; t += x.n_blocks) {
        const int b0 = (t % nb) * 64, d0 = (t / nb) * 64;
        for (int r = ty; r < 64; r += NTHREADS / 64)
            tile[r][tx] = (b0 + r < a.B) ? a.X[(int64_t)(b0 + r) * a.ldx + d0 + tx] : (uint16_t)0;
        __syncthreads();
        for (int r = ty; r < 64; r += NTHREADS / 64) x.XT[(int64_t)(d0 + r) * x.ldxt + b0 + tx] = tile[tx][r];
        __syncthreads();
    }
}

// dz of a thin tile: the same steps as in bwd_recompute_dz below on a 256-class x 64-row tile.  Its
// column sums are one db partial, in the slot the matching wave column of a full tile would fill.
__device__ __forceinline__ void dz_thin(const FcArgs& a, const TileRef& r, char* lds,
                                        const float* __restrict__ logsumexp, float grad_scale,
                                        uint16_t* __restrict__ dZ, int64_t ldz, float* __restrict__ db_part) {
    float* sbias = reinterpret_cast<float*>(lds);
    thin_acc_t acc;
    logits_thin(acc, a, r.ct, r.bt, r.piece, lds, sbias);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, jl = lane & 15;
    const int cw0 = r.ct * TILE_M + wave * THIN_WAVE_M;
    const int row0 = r.bt * TILE_N + r.piece * THIN_N;
#pragma unroll
    for (int nt = 0; nt < THIN_NT; ++nt) {
        const int row = row0 + 16 * nt + jl;
        const bool row_ok = row < a.B;
        const float lse = row_ok ? logsumexp[row] : 0.0f;
        const float gs = row_ok ? grad_scale : 0.0f;
        const float shift = __log2f(fabsf(gs)) - lse * LOG2E;
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[mt][nt][v] = __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][v], LOG2E, shift));
        if (grad_scale < 0.0f) {
#pragma unroll
            for (int mt = 0; mt < THIN_MT; ++mt) acc[mt][nt] = -acc[mt][nt];
        }
        const int local = row_ok ? a.labels[row] - a.class_offset : -1;
        const bool in_shard = local >= 0 && local < a.C;
        const int rel = local - cw0;
        const bool mine = in_shard && rel >= 0 && rel < THIN_WAVE_M && ((rel & 15) >> 2) == g;
        if (__any(mine)) {
#pragma unroll
            for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (mine && acc_row(mt, v, g) == rel) acc[mt][nt][v] -= gs;
        }
    }
    if (db_part != nullptr) {
        // a lane adds its four N-tiles; the 16 lanes with the same classes reduce-scatter the 8 sums in
        // three exchange steps and add the last pair, so lanes 2 i and 2 i + 1 both hold sum i
        float val[4 * THIN_MT];
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                val[4 * mt + v] = (acc[mt][0][v] + acc[mt][1][v]) + (acc[mt][2][v] + acc[mt][3][v]);
#pragma unroll
        for (int step = 0; step < 3; ++step) {
            const int h = (2 * THIN_MT) >> step, mask = 8 >> step;
            const bool up = (jl & mask) != 0;
#pragma unroll
            for (int i = 0; i < h; ++i) {
                const float keep = up ? val[i + h] : val[i];
                const float send = up ? val[i] : val[i + h];
                val[i] = keep + lane_xor(send, mask);
            }
        }
        val[0] += lane_xor(val[0], 1);
        if ((jl & 1) == 0) {
            const int i = jl >> 1;                      // accumulator row index 4 * mt + v
            db_part[(int64_t)(4 * r.bt + r.piece) * ldz + cw0 + 16 * (i >> 2) + 4 * g + (i & 3)] = val[0];
        }
    }
    __syncthreads();                       // the bias staging area is about to be overwritten
#pragma unroll
    for (int nt = 0; nt < THIN_NT; ++nt) {
        const int n = 16 * nt + jl;
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt) {
            u32x2 pk;
            pk[0] = pack_bf16(acc[mt][nt][0], acc[mt][nt][1]);
            pk[1] = pack_bf16(acc[mt][nt][2], acc[mt][nt][3]);
            *reinterpret_cast<u32x2*>(lds + out_tile_offset(n, wave * THIN_WAVE_M + 16 * mt + 4 * g)) = pk;
        }
    }
    __syncthreads();
    lds_tile_store_rows(lds, dZ + (int64_t)row0 * ldz + r.ct * TILE_M, ldz, THIN_N, TILE_M);
}

__global__ __launch_bounds__(NTHREADS) void bwd_recompute_dz(FcArgs a, const float* __restrict__ logsumexp,
                                                              float grad_scale, uint16_t* __restrict__ dZ,
                                                              int64_t ldz, float* __restrict__ db_part,
                                                              XtArgs xt) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    float* sbias = reinterpret_cast<float*>(lds);
    if ((int)blockIdx.x >= xt.first_block) {
        transpose_x_tiles(a, xt, (int)blockIdx.x - xt.first_block, lds);
        return;
    }
    const TileRef ref = logits_tile_ref(a);
    if (!ref.valid) return;
    if (ref.piece >= 0) {
        dz_thin(a, ref, lds, logsumexp, grad_scale, dZ, ldz, db_part);
        return;
    }
    const int ct = ref.ct, bt = ref.bt;

    acc_t acc;
    logits_tile(acc, a, ct, bt, lds, sbias);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
    const int cw0 = ct * TILE_M + wm * WAVE_M;

#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = bt * TILE_N + wn * WAVE_N + 16 * nt + jl;     // < Bpad: dZ has that many rows
        const bool row_ok = row < a.B;
        const float lse = row_ok ? logsumexp[row] : 0.0f;
        const float gs = row_ok ? grad_scale : 0.0f;                   // padded rows store exact zeros
        // |g| * exp(z - lse) = exp2(z * log2 e + (log2 |g| - lse * log2 e)): one FMA and one exp2 per
        // element; g = 0 gives a shift of -inf and exact zeros, as does z = -inf on padded classes.
        const float shift = __log2f(fabsf(gs)) - lse * LOG2E;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[mt][nt][v] = __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][v], LOG2E, shift));
        if (grad_scale < 0.0f) {                                        // uniform; the usual scales are positive
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = -acc[mt][nt];
        }

        const int local = row_ok ? a.labels[row] - a.class_offset : -1;
        const bool in_shard = local >= 0 && local < a.C;
        const int rel = local - cw0;
        const bool mine = in_shard && rel >= 0 && rel < WAVE_M && ((rel & 15) >> 2) == g;
        if (__any(mine)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (mine && acc_row(mt, v, g) == rel) acc[mt][nt][v] -= gs;
        }
    }

    // db: the tile's column sums over its batch rows, taken from the fp32 values.  A lane first adds
    // its four N-tiles, then the 16 lanes that hold the same classes reduce-scatter their 32 sums in
    // four exchange steps (16, 8, 4, 2 values sent), which leaves lane jl the sums of accumulator
    // rows 2 jl and 2 jl + 1 (row index = 4 * M-tile + register).  One partial per wave column:
    // db_part[4 * bt + wn][class].
    if (db_part != nullptr) {
        float val[4 * MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                val[4 * mt + v] = (acc[mt][0][v] + acc[mt][1][v]) + (acc[mt][2][v] + acc[mt][3][v]);
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int h = (2 * MT) >> step, mask = 8 >> step;
            const bool up = (jl & mask) != 0;
#pragma unroll
            for (int i = 0; i < h; ++i) {
                const float keep = up ? val[i + h] : val[i];
                const float send = up ? val[i] : val[i + h];
                val[i] = keep + lane_xor(send, mask);
            }
        }
        const int cls = cw0 + 16 * (jl >> 1) + 4 * g + 2 * (jl & 1);
        f32x2 two = {val[0], val[1]};
        *reinterpret_cast<f32x2*>(db_part + (int64_t)(4 * bt + wn) * ldz + cls) = two;
    }

    // dz [row][class] feeds both the dX contraction (over classes, read along its rows) and the dW
    // contraction (over rows, read across them).  The tile is staged in LDS so that it leaves in
    // whole 512-byte rows.
    __syncthreads();                       // the bias staging area is about to be overwritten
    acc_to_lds_bf16(acc, lds);
    __syncthreads();
    lds_tile_store_rows(lds, dZ + (int64_t)bt * TILE_N * ldz + ct * TILE_M, ldz, TILE_N, TILE_M);
}

// Predictions of the shard: P[i][c] = exp(z[i][c] - lse[i]) as bf16, the same GEMM and staging as
// bwd_recompute_dz without the one-hot term, written straight into the caller's [B][ldp] matrix
// (ragged edges cut at B and C).
__global__ __launch_bounds__(NTHREADS) void predict_probs(FcArgs a, const float* __restrict__ logsumexp,
                                                           uint16_t* __restrict__ P, int64_t ldp) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    float* sbias = reinterpret_cast<float*>(lds);
    const int tile = xcd_logical_tile(a.nBT * a.nCT);
    if (tile < 0) return;
    const int ct = tile / a.nBT, bt = tile % a.nBT;

    acc_t acc;
    logits_tile(acc, a, ct, bt, lds, sbias);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 3, jl = lane & 15;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int row = bt * TILE_N + wn * WAVE_N + 16 * nt + jl;
        const float shift = row < a.B ? -logsumexp[row] * LOG2E : 0.0f;      // rows beyond B are not stored
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[mt][nt][v] = __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][v], LOG2E, shift));
    }
    __syncthreads();                       // the bias staging area is about to be overwritten
    acc_to_lds_bf16(acc, lds);
    __syncthreads();
    const int b_left = a.B - bt * TILE_N, c_left = a.C - ct * TILE_M;
    lds_tile_store_rows(lds, P + (int64_t)bt * TILE_N * ldp + ct * TILE_M, ldp, b_left < TILE_N ? b_left : TILE_N,
                        c_left < TILE_M ? c_left : TILE_M);
}

// ---- arg-max predictions --------------------------------------------------------------------------
// The better of two (logit, class) candidates: the larger logit, the lower class id among equals.
__device__ __forceinline__ void better_of(float& v, int& c, float v2, int c2) {
    if (v2 > v || (v2 == v && c2 < c)) {
        v = v2;
        c = c2;
    }
}

// Top-1 of every row over one 256-class tile: the logits GEMM of fwd_logits_stats with an arg-max
// epilogue.  Partial (logit, shard-local class) pairs go to part_val / part_cls [class tile][row].
__global__ __launch_bounds__(NTHREADS) void top1_logits(FcArgs a, float* __restrict__ part_val,
                                                         int* __restrict__ part_cls) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    float* sbias = reinterpret_cast<float*>(lds);
    float* red_v = sbias + 256;                              // [2][256]
    int* red_c = reinterpret_cast<int*>(red_v + 512);
    const int tile = xcd_logical_tile(a.nBT * a.nCT);
    if (tile < 0) return;
    const int ct = tile / a.nBT, bt = tile % a.nBT;
    acc_t acc;
    logits_tile(acc, a, ct, bt, lds, sbias);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
    const int cw0 = ct * TILE_M + wm * WAVE_M;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float best = NEG_INF;
        int cls = INT_MAX;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (acc[mt][nt][v] > best) {                 // classes are visited in increasing order
                    best = acc[mt][nt][v];
                    cls = cw0 + acc_row(mt, v, g);
                }
        better_of(best, cls, lane_xor(best, 16), __shfl_xor(cls, 16, 64));
        better_of(best, cls, lane_xor(best, 32), __shfl_xor(cls, 32, 64));
        if (g == 0) {
            red_v[wm * 256 + wn * WAVE_N + 16 * nt + jl] = best;
            red_c[wm * 256 + wn * WAVE_N + 16 * nt + jl] = cls;
        }
    }
    __syncthreads();
    if (tid < 256) {
        float v = red_v[tid];
        int c = red_c[tid];
        better_of(v, c, red_v[256 + tid], red_c[256 + tid]);
        const int64_t o = (int64_t)ct * a.Bpad + bt * TILE_N + tid;
        part_val[o] = v;
        part_cls[o] = c;
    }
}

// Merges candidates of one row: n candidates `stride` apart; `base` is added to the winning class.
// One thread per row (the candidate lists are a few hundred entries of a few MB in total).
__global__ __launch_bounds__(256) void merge_top1(const float* __restrict__ val, const int* __restrict__ cls, int n,
                                                  int64_t stride, int B, int base, float* __restrict__ out_val,
                                                  int* __restrict__ out_cls) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    float v = NEG_INF;
    int c = INT_MAX;
    for (int t = 0; t < n; ++t) better_of(v, c, val[t * stride + i], cls[t * stride + i]);
    out_val[i] = v;
    out_cls[i] = c == INT_MAX ? c : c + base;
}

struct DxArgs {
    const uint16_t* dZ; int64_t ldz;     // [Bpad][Cpad]
    const uint16_t* W; int64_t ldw;      // [C][D]
    int B, D, C;
    int Bpad;
    int nDT, nBT, splits, steps_per_split, steps_total;
    float* out; int64_t ldo; int64_t split_stride;   // out[split][b][d]
};

// dX tile: M = batch rows (A = dz, k contiguous), N = features d (B operand = W_s read k-strided: the
// narrower side of a wave's sub-tile, so the slower transposing LDS reads are the fewer ones),
// K = the shard's classes, cut into `splits` ranges.
__global__ __launch_bounds__(NTHREADS) void bwd_dx(DxArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    const int tile = xcd_logical_tile(a.nDT * a.nBT * a.splits);
    if (tile < 0) return;
    // The 32 consecutive tiles that an XCD runs at a time should share their panels: up to four batch tiles, batch
    // tiles fastest (all tiles of 32 / nBT feature tiles); more, feature tiles fastest (the tiles that share a dz
    // panel, the larger operand, sit on one XCD).
    const int td = tile % (a.nBT * a.nDT), sp = tile / (a.nBT * a.nDT);
    const int bt = a.nBT <= 4 ? td % a.nBT : td / a.nDT;
    const int dt = a.nBT <= 4 ? td / a.nBT : td % a.nDT;
    const int s0 = sp * a.steps_per_split;
    int ns = a.steps_total - s0;
    ns = ns < a.steps_per_split ? ns : a.steps_per_split;

    acc_t acc;
    zero_acc(acc);
    const Operand A = make_operand(a.dZ, a.ldz, a.Bpad, a.ldz);
    const Operand Bo = make_operand(a.W, a.ldw, a.C, a.D);          // classes beyond the shard read as zeros
    gemm_mainloop<KC, KS>(acc, A, Bo, bt * TILE_M, dt * TILE_N, s0 * TILE_K, ns, lds);

    // The accumulator layout gives a lane four consecutive rows of one column: direct stores would be 64-byte
    // pieces.  Instead each half of the tile (the 128 rows of one wave row) goes through LDS as fp32
    // [128 rows][256 columns] (16-float chunks XOR-ed with (row >> 2) & 3, which spreads the four row groups of
    // a wave's store over the banks) and leaves in whole 1 KiB rows.
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
    float* out = a.out + sp * a.split_stride;
    float* tile_f32 = reinterpret_cast<float*>(lds);
    const int d_left = a.D - dt * TILE_N;
#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
        if (wm == h) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int col = wn * WAVE_N + 16 * nt + jl;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * mt + 4 * g + v;
                        tile_f32[row * 256 + ((((col >> 4) ^ ((row >> 2) & 3)) << 4) | (col & 15))] = acc[mt][nt][v];
                    }
            }
        }
        __syncthreads();
#pragma unroll 4
        for (int i = 0; i < 16; ++i) {
            const int q = tid + NTHREADS * i;
            const int row = q >> 6, c4 = q & 63;
            const int grow = bt * TILE_M + h * WAVE_M + row;
            if (grow < a.B && 4 * c4 < d_left) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(
                    tile_f32 + row * 256 + ((((c4 >> 2) ^ ((row >> 2) & 3)) << 4) | ((c4 & 3) << 2)));
                *reinterpret_cast<f32x4*>(out + (int64_t)grow * a.ldo + dt * TILE_N + 4 * c4) = v;
            }
        }
        __syncthreads();
    }
}

// The two small reductions that finish the backward call: the split-K partials of dX are summed in a
// fixed order (one float4 per thread and turn; optionally accumulating into the caller's dX), and the
// per-row-tile column sums into db.  Run by the workgroups of bwd_dw beyond its GEMM tiles (handed out
// last, onto compute units that the final, partial round of GEMM tiles leaves idle).
struct FinishArgs {
    const float* parts; int splits; int64_t split_stride;   // nullptr: dX was written directly
    int B, D;
    float* dX; int64_t lddx; int accumulate;
    const float* db_part; int n_db_parts; int64_t db_stride; // nullptr: no db wanted
    int C; float* db;
    int sgd; float lr;                                        // sgd: db is the bias, updated in place
    int first_block, n_blocks;
};

__device__ __forceinline__ void finish_bwd(const FinishArgs& f, int worker) {
    const int64_t stride = (int64_t)f.n_blocks * NTHREADS;
    const int64_t me = (int64_t)worker * NTHREADS + threadIdx.x;
    if (f.parts != nullptr) {
        const int d4 = f.D >> 2;
        const int64_t n4 = (int64_t)f.B * d4;
        for (int64_t i = me; i < n4; i += stride) {
            const int row = (int)(i / d4), d = (int)(i % d4) * 4;
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
            for (int p = 0; p < f.splits; ++p)
                s += *reinterpret_cast<const f32x4*>(f.parts + p * f.split_stride + (int64_t)row * f.D + d);
            float* o = f.dX + (int64_t)row * f.lddx + d;
            if (f.accumulate) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] += s[e];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = s[e];
            }
        }
    }
    if (f.db_part != nullptr) {
        for (int64_t c = me; c < f.C; c += stride) {
            float s = 0.0f;
            for (int t = 0; t < f.n_db_parts; ++t) s += f.db_part[t * f.db_stride + c];
            f.db[c] = f.sgd ? fmaf(-f.lr, s, f.db[c]) : s;
        }
    }
}

struct DwArgs {
    const uint16_t* XT; int64_t ldxt;    // [D][Bpad]
    const uint16_t* dZ; int64_t ldz;     // [Bpad][Cpad]
    int D, C, Bpad;
    int nDT, nCT, k_steps;
    uint16_t* dW; int64_t lddw;          // sgd: the weights themselves, updated in place
    int sgd; float lr;
    TilePlan plan;                       // full tiles, and the thin ones a ragged last round is cut into
};

// dW^T tile: M = features d (A = X^T, k contiguous), N = classes (B operand = dz read k-strided, the
// narrower side of a wave's sub-tile as in bwd_dx), K = batch rows.
// TRACE: thread 0 of the workgroup also writes the shader clock at six points of its tile, and which compute
// unit it ran on, to trace[8 * tile ..] (diagnostics; the arithmetic and the stores are the same).
template <bool TRACE>
__device__ __forceinline__ void dw_tile(const DwArgs& a, char* lds, unsigned long long* trace) {
    unsigned long long stamp[6];
    if (TRACE) stamp[0] = __builtin_readcyclecounter();
    const int tile = xcd_logical_tile(a.plan.n_full);
    if (tile < 0) return;
    const int dt = tile % a.nDT, ct = tile / a.nDT;    // feature tiles fastest: neighbours share the dz panel

    acc_t acc;
    zero_acc(acc);
    const Operand A = make_operand(a.XT, a.ldxt, a.D, a.ldxt);
    const Operand Bo = make_operand(a.dZ, a.ldz, a.Bpad, a.ldz);
    if (TRACE) stamp[1] = __builtin_readcyclecounter();
    // workgroups are dealt out 256 at a time, 32 to each XCD: alternate the direction round by round, so that a
    // compute unit's next tile finds the end of the X^T panels, which it has just read, still in the L2
    gemm_mainloop<KC, KS>(acc, A, Bo, dt * TILE_M, ct * TILE_N, 0, a.k_steps, lds, ((blockIdx.x >> 8) & 1) != 0);
    if (TRACE) stamp[2] = __builtin_readcyclecounter();

    // [class][feature] tile through LDS, then whole 512-byte rows of dW
    acc_to_lds_bf16(acc, lds);
    __syncthreads();
    if (TRACE) stamp[3] = __builtin_readcyclecounter();
    const int c_left = a.C - ct * TILE_N, d_left = a.D - dt * TILE_M;
    uint16_t* out = a.dW + (int64_t)ct * TILE_N * a.lddw + dt * TILE_M;
    const int n_valid = c_left < TILE_N ? c_left : TILE_N, m_valid = d_left < TILE_M ? d_left : TILE_M;
    if (a.sgd) lds_tile_update_rows(lds, out, a.lddw, n_valid, m_valid, a.lr);
    else lds_tile_store_rows(lds, out, a.lddw, n_valid, m_valid);
    if (TRACE) {
        stamp[4] = __builtin_readcyclecounter();
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this wave's stores have been acknowledged
        stamp[5] = __builtin_readcyclecounter();
        if (threadIdx.x == 0) {
            // hardware registers HW_ID (4: wave, SIMD, compute unit, shader array and engine) and XCC_ID (20)
            const unsigned long long hw = __builtin_amdgcn_s_getreg((31 << 11) | 4);
            const unsigned long long xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20);
            unsigned long long* t = trace + 8 * (int64_t)tile;
#pragma unroll
            for (int i = 0; i < 6; ++i) t[i] = stamp[i];
            t[6] = (unsigned long long)blockIdx.x;
            t[7] = (xcc << 32) | hw;
        }
    }
}

// Thin tile of dW: all 256 features of feature tile dt x 64 classes (piece 0 .. 3 of class tile ct); the dz
// operand is k-strided.  Used for the tiles of a ragged last round when the contraction is long (the host
// decides, plan_tiles); not traced.
__device__ __forceinline__ void dw_thin(const DwArgs& a, int q, char* lds) {
    const int tile = a.plan.n_full + (q >> 2), piece = q & 3;
    const int dt = tile % a.nDT, ct = tile / a.nDT;
    const int c0 = ct * TILE_N + piece * THIN_N;
    if (c0 >= a.C) return;                              // a piece entirely beyond the shard's classes
    thin_acc_t acc;
#pragma unroll
    for (int i = 0; i < THIN_MT; ++i)
#pragma unroll
        for (int j = 0; j < THIN_NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const Operand A = make_operand(a.XT, a.ldxt, a.D, a.ldxt);
    const Operand Bo = make_operand(a.dZ, a.ldz, a.Bpad, a.ldz);
    thin_mainloop<KS>(acc, A, Bo, dt * TILE_M, c0, 0, a.k_steps, lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, jl = lane & 15;
#pragma unroll
    for (int nt = 0; nt < THIN_NT; ++nt) {
        const int n = 16 * nt + jl;
#pragma unroll
        for (int mt = 0; mt < THIN_MT; ++mt) {
            u32x2 pk;
            pk[0] = pack_bf16(acc[mt][nt][0], acc[mt][nt][1]);
            pk[1] = pack_bf16(acc[mt][nt][2], acc[mt][nt][3]);
            *reinterpret_cast<u32x2*>(lds + out_tile_offset(n, wave * THIN_WAVE_M + 16 * mt + 4 * g)) = pk;
        }
    }
    __syncthreads();
    const int c_left = a.C - c0, d_left = a.D - dt * TILE_M;
    uint16_t* out = a.dW + (int64_t)c0 * a.lddw + dt * TILE_M;
    const int n_valid = c_left < THIN_N ? c_left : THIN_N, m_valid = d_left < TILE_M ? d_left : TILE_M;
    if (a.sgd) lds_tile_update_rows(lds, out, a.lddw, n_valid, m_valid, a.lr);
    else lds_tile_store_rows(lds, out, a.lddw, n_valid, m_valid);
}

__global__ __launch_bounds__(NTHREADS) void bwd_dw(DwArgs a, FinishArgs fin) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    if ((int)blockIdx.x >= fin.first_block) {
        finish_bwd(fin, (int)blockIdx.x - fin.first_block);
        return;
    }
    if ((int)blockIdx.x >= a.plan.thin_first) {
        dw_thin(a, (int)blockIdx.x - a.plan.thin_first, lds);
        return;
    }
    dw_tile<false>(a, lds, nullptr);
}

__global__ __launch_bounds__(NTHREADS) void bwd_dw_traced(DwArgs a, FinishArgs fin, unsigned long long* trace) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    if ((int)blockIdx.x >= fin.first_block) {
        finish_bwd(fin, (int)blockIdx.x - fin.first_block);
        return;
    }
    if ((int)blockIdx.x >= a.plan.thin_first) {
        dw_thin(a, (int)blockIdx.x - a.plan.thin_first, lds);
        return;
    }
    dw_tile<true>(a, lds, trace);
}

// ---- host side -----------------------------------------------------------------------------------

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
static inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline int xcd_grid(int n_tiles) { return 8 * ((n_tiles + 7) / 8); }

// Full tiles fill whole rounds of the 256 compute units; a last round that would leave half of them or
// more idle is run as thin tiles (four per full tile) instead.
static TilePlan plan_tiles(int n_tiles, bool allow_thin) {
    TilePlan t;
    const int tail = n_tiles % 256;
    const bool thin = allow_thin && tail > 0 && tail <= 128;
    t.n_full = thin ? n_tiles - tail : n_tiles;
    t.n_thin = thin ? 4 * tail : 0;
    t.thin_first = xcd_grid(t.n_full);
    return t;
}
// Shortest contraction (k-steps of 64 batch rows) for which the dW kernel cuts the tiles of a ragged last round
// into thin ones: measured slower at 16 k-steps (the last round is mostly output there), faster at 128.
static const int DW_THIN_MIN_K_STEPS = 48;
// Workgroups appended to a GEMM launch for its small side job (X^T, the final reductions).
static const int SIDE_BLOCKS = 128;

struct BwdPlan {
    int64_t Bpad, Cpad;
    int nBT, nCT, nDT;
    int steps_total, splits, steps_per_split;
    size_t dz_bytes, xt_bytes, dbp_bytes, parts_bytes;
};

static bool shape_ok(int32_t B, int32_t D, int32_t C) { return B > 0 && D > 0 && C > 0 && D % 64 == 0; }

// The kernels address an operand with 32-bit byte offsets, tiles may hang 256 rows over its end.
static bool fits_32bit_offsets(int64_t rows, int64_t ld) { return (rows + 256) * ld * 2 < ((int64_t)1 << 32); }

static BwdPlan plan_bwd(int32_t B, int32_t D, int32_t C) {
    BwdPlan p;
    p.Bpad = round_up(B, 256);
    p.Cpad = round_up(C, 256);
    p.nBT = (int)(p.Bpad / 256);
    p.nCT = (int)(p.Cpad / 256);
    p.nDT = (int)(round_up(D, 256) / 256);
    p.steps_total = (int)(round_up(C, TILE_K) / TILE_K);
    const int tiles = p.nDT * p.nBT;
    int want = tiles >= 256 ? 1 : (256 + tiles - 1) / tiles;     // fill the 256 CUs once
    if (want > p.steps_total) want = p.steps_total;
    p.steps_per_split = (p.steps_total + want - 1) / want;
    p.splits = (p.steps_total + p.steps_per_split - 1) / p.steps_per_split;
    p.dz_bytes = (size_t)p.Bpad * p.Cpad * 2;
    p.xt_bytes = (size_t)D * p.Bpad * 2;
    p.dbp_bytes = (size_t)4 * p.nBT * p.Cpad * 4;        // one db partial per 64-row wave column
    p.parts_bytes = (size_t)p.splits * B * D * 4;
    return p;
}

static size_t fwd_bytes(int32_t B, int32_t C) {
    return (size_t)2 * (round_up(C, 256) / 256) * round_up(B, 256) * sizeof(float);
}

static int check_fc_common(const void* X, int64_t ldx, const void* W, int64_t ldw, const float* bias,
                           const int32_t* labels, int32_t B, int32_t D, int32_t C, int32_t class_offset) {
    if (!X || !W || !labels) return WS_ERR_NULL;
    if (!shape_ok(B, D, C)) return WS_ERR_SHAPE;
    if (ldx < D || ldw < D) return WS_ERR_SHAPE;
    if (!fits_32bit_offsets(B, ldx) || !fits_32bit_offsets(C, ldw)) return WS_ERR_SHAPE;
    if (class_offset < 0 || (int64_t)class_offset + C > INT32_MAX) return WS_ERR_RANGE;
    if (!aligned(X, 16) || !aligned(W, 16) || ldx % 8 || ldw % 8) return WS_ERR_ALIGN;
    if (!aligned(labels, 4) || (bias && !aligned(bias, 4))) return WS_ERR_ALIGN;
    return WS_OK;
}


// ---- built-in scratch of the entry point that allocates nothing ---------------------------------------
// A fixed array in the code object stands in for the forward call's workspace.  Every GPU the library
// runs on holds its own copy at its own address; in host code the array's name is only a handle, so the
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[WS_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device (looked up at the first call on that device).
static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return WS_ERR_HIP;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return WS_ERR_HIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return WS_OK;
}

// ---- optional per-kernel timing --------------------------------------------------------------------
// When enabled, every kernel launch is bracketed by a pair of events recorded on the launch stream.
// The pairs come from a pool created by ws_profile_enable; when the pool is used up, launches go
// untimed.  Not thread safe; meant for benchmarks.
enum KernelId { KID_FWD = 0, KID_MERGE, KID_COMBINE, KID_MEAN, KID_DZ, KID_DX, KID_DW, KID_PREDICT, KID_TOP1, KID_TOP1_MERGE, KID_COUNT };
static const char* const kKernelNames[KID_COUNT] = {"fwd_logits_stats", "merge_class_tiles", "combine_partials",
                                                    "mean_loss", "bwd_recompute_dz", "bwd_dx", "bwd_dw",
                                                    "predict_probs", "top1_logits", "merge_top1"};
struct ProfState {
    bool on = false;
    bool paused = false;
    int capacity = 0, used = 0;
    hipEvent_t* start = nullptr;
    hipEvent_t* stop = nullptr;
    int* kid = nullptr;
};
static ProfState g_prof;

// ws_profile_trace_dw: where the dW kernel of the following backward calls writes its per-tile clock stamps.
static unsigned long long* g_dw_trace = nullptr;
static int64_t g_dw_trace_tiles = 0;

struct ScopedTimer {
    int slot = -1;
    hipStream_t s;
    ScopedTimer(int kid, hipStream_t stream) : s(stream) {
        if (g_prof.on && !g_prof.paused && g_prof.used < g_prof.capacity) {
            slot = g_prof.used++;
            g_prof.kid[slot] = kid;
            (void)hipEventRecord(g_prof.start[slot], s);
        }
    }
    ~ScopedTimer() {
        if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s);
    }
};
#define WS_LAUNCH(kid, kernel, grid, block, stream, ...)                         \
    do {                                                                         \
        ScopedTimer timer_(kid, stream);                                         \
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);         \
    } while (0)

static int launch_status() { return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP; }

}  // namespace ws

using namespace ws;

extern "C" {

const char* ws_status_string(int status) {
    switch (status) {
        case WS_OK: return "WS_OK";
        case WS_ERR_NULL: return "WS_ERR_NULL";
        case WS_ERR_SHAPE: return "WS_ERR_SHAPE";
        case WS_ERR_ALIGN: return "WS_ERR_ALIGN";
        case WS_ERR_RANGE: return "WS_ERR_RANGE";
        case WS_ERR_WORKSPACE: return "WS_ERR_WORKSPACE";
        case WS_ERR_HIP: return "WS_ERR_HIP";
        case WS_ERR_LIMIT: return "WS_ERR_LIMIT";
        default: return "WS_ERR_UNKNOWN";
    }
}

int ws_version(void) { return 1215; }

size_t ws_fwd_workspace_bytes(int32_t B, int32_t D, int32_t C_shard) {
    return shape_ok(B, D, C_shard) ? fwd_bytes(B, C_shard) : 0;
}

size_t ws_bwd_workspace_bytes(int32_t B, int32_t D, int32_t C_shard) {
    if (!shape_ok(B, D, C_shard)) return 0;
    const BwdPlan p = plan_bwd(B, D, C_shard);
    return p.dz_bytes + p.xt_bytes + p.dbp_bytes + p.parts_bytes;
}

// Argument checks of the forward call that do not concern the workspace.
static int check_fwd(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                     const int32_t* labels, int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                     float* row_max, float* row_sumexp, float* label_logit) {
    if (!row_max || !row_sumexp || !label_logit) return WS_ERR_NULL;
    int st = check_fc_common(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset);
    if (st != WS_OK) return st;
    if (!aligned(row_max, 4) || !aligned(row_sumexp, 4) || !aligned(label_logit, 4)) return WS_ERR_ALIGN;
    return WS_OK;
}

// Launches of the forward call; `workspace` holds fwd_bytes(B, C_shard) bytes, 16-byte aligned.
static int launch_fwd(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                      const int32_t* labels, int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                      float* row_max, float* row_sumexp, float* label_logit, void* workspace, void* stream) {
    FcArgs a;
    a.last_tile_first = 0;
    a.X = static_cast<const uint16_t*>(X); a.ldx = ldx;
    a.W = static_cast<const uint16_t*>(W_shard); a.ldw = ldw;
    a.bias = b_shard; a.labels = labels;
    a.B = B; a.D = D; a.C = C_shard; a.class_offset = class_offset;
    a.Bpad = (int)round_up(B, 256);
    a.nBT = a.Bpad / 256;
    a.nCT = (int)(round_up(C_shard, 256) / 256);
    float* part_max = static_cast<float*>(workspace);
    float* part_sum = part_max + (size_t)a.nCT * a.Bpad;
    hipStream_t s = static_cast<hipStream_t>(stream);
    a.plan = plan_tiles(a.nBT * a.nCT, true);
    WS_LAUNCH(KID_FWD, fwd_logits_stats, dim3(a.plan.thin_first + a.plan.n_thin), dim3(NTHREADS), s, a, part_max,
                       part_sum, label_logit);
    WS_LAUNCH(KID_MERGE, merge_class_tiles, dim3((B + 15) / 16), dim3(1024), s, part_max, part_sum, a.nCT,
                       a.Bpad, B, row_max, row_sumexp);
    return launch_status();
}

int ws_split_fc_fwd(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                    const int32_t* labels, int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                    float* row_max, float* row_sumexp, float* label_logit, void* workspace,
                    size_t workspace_bytes, void* stream) {
    int st = check_fwd(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset, row_max, row_sumexp,
                       label_logit);
    if (st != WS_OK) return st;
    if (!workspace || workspace_bytes < fwd_bytes(B, C_shard)) return WS_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return WS_ERR_ALIGN;
    return launch_fwd(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset, row_max, row_sumexp,
                      label_logit, workspace, stream);
}

int ws_split_fc_fwd_static(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                           const int32_t* labels, int32_t B, int32_t D, int32_t C_shard, int32_t class_offset,
                           float* row_max, float* row_sumexp, float* label_logit, void* stream) {
    int st = check_fwd(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset, row_max, row_sumexp,
                       label_logit);
    if (st != WS_OK) return st;
    if (fwd_bytes(B, C_shard) > (size_t)WS_STATIC_SCRATCH_BYTES) return WS_ERR_LIMIT;
    void* ws_ptr = nullptr;
    st = static_scratch(&ws_ptr);
    if (st != WS_OK) return st;
    // every partial the merge reads is written by the logits kernel of the same call: nothing to clear
    return launch_fwd(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset, row_max, row_sumexp,
                      label_logit, ws_ptr, stream);
}

int ws_combine_partials(const float* row_max, const float* row_sumexp, const float* label_logit, int32_t S,
                        int32_t B, int64_t shard_stride, float* logsumexp, float* loss_rows, float* loss_mean,
                        void* stream) {
    if (!row_max || !row_sumexp || !label_logit || !logsumexp || !loss_rows) return WS_ERR_NULL;
    if (B <= 0 || shard_stride < B) return WS_ERR_SHAPE;
    if (S < 1 || S > 65536) return WS_ERR_RANGE;
    if (!aligned(row_max, 4) || !aligned(row_sumexp, 4) || !aligned(label_logit, 4) || !aligned(logsumexp, 4) ||
        !aligned(loss_rows, 4) || (loss_mean && !aligned(loss_mean, 4)))
        return WS_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    WS_LAUNCH(KID_COMBINE, combine_partials_kernel, dim3((B + 255) / 256), dim3(256), s, row_max, row_sumexp,
                       label_logit, S, B, shard_stride, logsumexp, loss_rows);
    if (loss_mean) WS_LAUNCH(KID_MEAN, mean_loss_kernel, dim3(1), dim3(1024), s, loss_rows, B, loss_mean);
    return launch_status();
}

// The backward call.  sgd = 0: dW_shard / db_shard receive the gradients.  sgd = 1: dW_shard is the weight
// matrix itself (== W_shard) and db_shard the bias itself (== b_shard or NULL); both are updated in place
// by the last kernel, after every kernel that reads them.
static int run_bwd(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                   const float* logsumexp, const int32_t* labels, int32_t B, int32_t D, int32_t C_shard,
                   int32_t class_offset, float grad_scale, float* dX_partial, int64_t lddx,
                   int32_t accumulate_dx, void* dW_shard, int64_t lddw, float* db_shard, void* workspace,
                   size_t workspace_bytes, void* stream, int sgd, float lr) {
    if (!logsumexp || !dX_partial || !dW_shard) return WS_ERR_NULL;
    int st = check_fc_common(X, ldx, W_shard, ldw, b_shard, labels, B, D, C_shard, class_offset);
    if (st != WS_OK) return st;
    if (lddx < D || lddw < D) return WS_ERR_SHAPE;
    if (!aligned(dX_partial, 16) || !aligned(dW_shard, 16) || lddx % 4 || lddw % 8) return WS_ERR_ALIGN;
    if (!aligned(logsumexp, 4) || (db_shard && !aligned(db_shard, 4))) return WS_ERR_ALIGN;
    const BwdPlan p = plan_bwd(B, D, C_shard);
    if (!fits_32bit_offsets(p.Bpad, p.Cpad) || !fits_32bit_offsets(D, p.Bpad))
        return WS_ERR_SHAPE;
    if (!workspace || workspace_bytes < p.dz_bytes + p.xt_bytes + p.dbp_bytes + p.parts_bytes) return WS_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return WS_ERR_ALIGN;
    if (g_dw_trace != nullptr && (int64_t)p.nDT * p.nCT > g_dw_trace_tiles) return WS_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint16_t* dZ = static_cast<uint16_t*>(workspace);
    uint16_t* XT = dZ + (size_t)p.Bpad * p.Cpad;
    float* db_part = reinterpret_cast<float*>(static_cast<char*>(workspace) + p.dz_bytes + p.xt_bytes);
    float* parts = db_part + (size_t)4 * p.nBT * p.Cpad;

    FcArgs a;
    a.last_tile_first = 1;   // the forward call has just read the last class tiles of W: they may still be in the Infinity Cache
    a.X = static_cast<const uint16_t*>(X); a.ldx = ldx;
    a.W = static_cast<const uint16_t*>(W_shard); a.ldw = ldw;
    a.bias = b_shard; a.labels = labels;
    a.B = B; a.D = D; a.C = C_shard; a.class_offset = class_offset;
    a.Bpad = (int)p.Bpad; a.nBT = p.nBT; a.nCT = p.nCT;
    XtArgs xt;
    xt.XT = XT; xt.ldxt = p.Bpad;
    a.plan = plan_tiles(p.nBT * p.nCT, true);
    xt.first_block = a.plan.thin_first + a.plan.n_thin;
    xt.n_blocks = (int)std::min<int64_t>((p.Bpad / 64) * (D / 64), SIDE_BLOCKS);
    WS_LAUNCH(KID_DZ, bwd_recompute_dz, dim3(xt.first_block + xt.n_blocks), dim3(NTHREADS), s, a, logsumexp,
              grad_scale, dZ, p.Cpad, db_shard ? db_part : nullptr, xt);

    DxArgs x;
    x.dZ = dZ; x.ldz = p.Cpad; x.W = a.W; x.ldw = ldw;
    x.B = B; x.D = D; x.C = C_shard; x.Bpad = (int)p.Bpad;
    x.nDT = p.nDT; x.nBT = p.nBT; x.splits = p.splits; x.steps_per_split = p.steps_per_split;
    x.steps_total = p.steps_total;
    const bool direct = p.splits == 1 && !accumulate_dx;
    x.out = direct ? dX_partial : parts;
    x.ldo = direct ? lddx : D;
    x.split_stride = (int64_t)B * D;
    WS_LAUNCH(KID_DX, bwd_dx, dim3(xcd_grid(p.nDT * p.nBT * p.splits)), dim3(NTHREADS), s, x);
    DwArgs w;
    w.XT = XT; w.ldxt = p.Bpad; w.dZ = dZ; w.ldz = p.Cpad;
    w.D = D; w.C = C_shard; w.Bpad = (int)p.Bpad;
    w.nDT = p.nDT; w.nCT = p.nCT; w.k_steps = (B + TILE_K - 1) / TILE_K;
    w.dW = static_cast<uint16_t*>(dW_shard); w.lddw = lddw;
    w.sgd = sgd; w.lr = lr;
    // thin tiles pay off only where a tile is long: with few k-steps the last round is mostly output
    w.plan = plan_tiles(p.nDT * p.nCT, w.k_steps >= DW_THIN_MIN_K_STEPS);
    FinishArgs f;
    f.parts = direct ? nullptr : parts; f.splits = p.splits; f.split_stride = (int64_t)B * D;
    f.B = B; f.D = D; f.dX = dX_partial; f.lddx = lddx; f.accumulate = accumulate_dx;
    f.db_part = db_shard ? db_part : nullptr; f.n_db_parts = 4 * p.nBT; f.db_stride = p.Cpad;
    f.C = C_shard; f.db = db_shard;
    f.sgd = sgd; f.lr = lr;
    f.first_block = w.plan.thin_first + w.plan.n_thin;
    f.n_blocks = (f.parts || f.db_part) ? SIDE_BLOCKS : 0;
    if (g_dw_trace != nullptr) {
        WS_LAUNCH(KID_DW, bwd_dw_traced, dim3(f.first_block + f.n_blocks), dim3(NTHREADS), s, w, f, g_dw_trace);
    } else {
        WS_LAUNCH(KID_DW, bwd_dw, dim3(f.first_block + f.n_blocks), dim3(NTHREADS), s, w, f);
    }
    return launch_status();
}

int ws_split_fc_bwd(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                    const float* logsumexp, const int32_t* labels, int32_t B, int32_t D, int32_t C_shard,
                    int32_t class_offset, float grad_scale, float* dX_partial, int64_t lddx,
                    int32_t accumulate_dx, void* dW_shard, int64_t lddw, float* db_shard, void* workspace,
                    size_t workspace_bytes, void* stream) {
    return run_bwd(X, ldx, W_shard, ldw, b_shard, logsumexp, labels, B, D, C_shard, class_offset, grad_scale,
                   dX_partial, lddx, accumulate_dx, dW_shard, lddw, db_shard, workspace, workspace_bytes, stream, 0,
                   0.0f);
}

int ws_split_fc_bwd_sgd(const void* X, int64_t ldx, void* W_shard, int64_t ldw, float* b_shard,
                        const float* logsumexp, const int32_t* labels, int32_t B, int32_t D, int32_t C_shard,
                        int32_t class_offset, float grad_scale, float lr, float* dX_partial, int64_t lddx,
                        int32_t accumulate_dx, void* workspace, size_t workspace_bytes, void* stream) {
    if (!(lr == lr) || lr - lr != 0.0f) return WS_ERR_RANGE;          // NaN or infinite learning rate
    return run_bwd(X, ldx, W_shard, ldw, b_shard, logsumexp, labels, B, D, C_shard, class_offset, grad_scale,
                   dX_partial, lddx, accumulate_dx, W_shard, ldw, b_shard, workspace, workspace_bytes, stream, 1, lr);
}

int ws_split_fc_predict(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard,
                        const float* logsumexp, int32_t B, int32_t D, int32_t C_shard, void* P, int64_t ldp,
                        void* stream) {
    if (!X || !W_shard || !logsumexp || !P) return WS_ERR_NULL;
    if (!shape_ok(B, D, C_shard)) return WS_ERR_SHAPE;
    if (ldx < D || ldw < D || ldp < C_shard) return WS_ERR_SHAPE;
    if (!fits_32bit_offsets(B, ldx) || !fits_32bit_offsets(C_shard, ldw)) return WS_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(W_shard, 16) || !aligned(P, 16) || ldx % 8 || ldw % 8 || ldp % 8) return WS_ERR_ALIGN;
    if (!aligned(logsumexp, 4) || (b_shard && !aligned(b_shard, 4))) return WS_ERR_ALIGN;
    FcArgs a;
    a.last_tile_first = 0;
    a.X = static_cast<const uint16_t*>(X); a.ldx = ldx;
    a.W = static_cast<const uint16_t*>(W_shard); a.ldw = ldw;
    a.bias = b_shard; a.labels = nullptr;
    a.B = B; a.D = D; a.C = C_shard; a.class_offset = 0;
    a.Bpad = (int)round_up(B, 256);
    a.nBT = a.Bpad / 256;
    a.nCT = (int)(round_up(C_shard, 256) / 256);
    a.plan = plan_tiles(a.nBT * a.nCT, false);
    hipStream_t s = static_cast<hipStream_t>(stream);
    WS_LAUNCH(KID_PREDICT, predict_probs, dim3(xcd_grid(a.nBT * a.nCT)), dim3(NTHREADS), s, a, logsumexp,
              static_cast<uint16_t*>(P), ldp);
    return launch_status();
}

int ws_split_fc_top1(const void* X, int64_t ldx, const void* W_shard, int64_t ldw, const float* b_shard, int32_t B,
                     int32_t D, int32_t C_shard, int32_t class_offset, float* top_logit, int32_t* top_class,
                     void* workspace, size_t workspace_bytes, void* stream) {
    if (!X || !W_shard || !top_logit || !top_class) return WS_ERR_NULL;
    if (!shape_ok(B, D, C_shard)) return WS_ERR_SHAPE;
    if (ldx < D || ldw < D) return WS_ERR_SHAPE;
    if (!fits_32bit_offsets(B, ldx) || !fits_32bit_offsets(C_shard, ldw)) return WS_ERR_SHAPE;
    if (class_offset < 0 || (int64_t)class_offset + C_shard > INT32_MAX) return WS_ERR_RANGE;
    if (!aligned(X, 16) || !aligned(W_shard, 16) || ldx % 8 || ldw % 8) return WS_ERR_ALIGN;
    if (!aligned(top_logit, 4) || !aligned(top_class, 4) || (b_shard && !aligned(b_shard, 4))) return WS_ERR_ALIGN;
    if (!workspace || workspace_bytes < fwd_bytes(B, C_shard)) return WS_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return WS_ERR_ALIGN;
    FcArgs a;
    a.last_tile_first = 0;
    a.X = static_cast<const uint16_t*>(X); a.ldx = ldx;
    a.W = static_cast<const uint16_t*>(W_shard); a.ldw = ldw;
    a.bias = b_shard; a.labels = nullptr;
    a.B = B; a.D = D; a.C = C_shard; a.class_offset = class_offset;
    a.Bpad = (int)round_up(B, 256);
    a.nBT = a.Bpad / 256;
    a.nCT = (int)(round_up(C_shard, 256) / 256);
    a.plan = plan_tiles(a.nBT * a.nCT, false);
    float* part_val = static_cast<float*>(workspace);
    int* part_cls = reinterpret_cast<int*>(part_val + (size_t)a.nCT * a.Bpad);
    hipStream_t s = static_cast<hipStream_t>(stream);
    WS_LAUNCH(KID_TOP1, top1_logits, dim3(xcd_grid(a.nBT * a.nCT)), dim3(NTHREADS), s, a, part_val, part_cls);
    WS_LAUNCH(KID_TOP1_MERGE, merge_top1, dim3((B + 255) / 256), dim3(256), s, part_val, part_cls, a.nCT,
              (int64_t)a.Bpad, B, class_offset, top_logit, top_class);
    return launch_status();
}

int ws_combine_top1(const float* top_logit, const int32_t* top_class, int32_t S, int32_t B, int64_t shard_stride,
                    float* best_logit, int32_t* best_class, void* stream) {
    if (!top_logit || !top_class || !best_logit || !best_class) return WS_ERR_NULL;
    if (B <= 0 || shard_stride < B) return WS_ERR_SHAPE;
    if (S < 1 || S > 65536) return WS_ERR_RANGE;
    if (!aligned(top_logit, 4) || !aligned(top_class, 4) || !aligned(best_logit, 4) || !aligned(best_class, 4))
        return WS_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    WS_LAUNCH(KID_TOP1_MERGE, merge_top1, dim3((B + 255) / 256), dim3(256), s, top_logit, top_class, S, shard_stride,
              B, 0, best_logit, best_class);
    return launch_status();
}

static void profile_free_pool() {
    for (int i = 0; i < g_prof.capacity; ++i) {
        (void)hipEventDestroy(g_prof.start[i]);
        (void)hipEventDestroy(g_prof.stop[i]);
    }
    delete[] g_prof.start; delete[] g_prof.stop; delete[] g_prof.kid;
    g_prof = ProfState();
}

int ws_profile_enable(int32_t max_launches) {
    if (g_prof.start) profile_free_pool();
    if (max_launches <= 0) return WS_OK;
    g_prof.start = new hipEvent_t[max_launches];
    g_prof.stop = new hipEvent_t[max_launches];
    g_prof.kid = new int[max_launches];
    for (int i = 0; i < max_launches; ++i) {
        if (hipEventCreate(&g_prof.start[i]) != hipSuccess) {
            profile_free_pool();                      // the pairs created so far; timing stays off
            return WS_ERR_HIP;
        }
        if (hipEventCreate(&g_prof.stop[i]) != hipSuccess) {
            (void)hipEventDestroy(g_prof.start[i]);
            profile_free_pool();
            return WS_ERR_HIP;
        }
        g_prof.capacity = i + 1;
    }
    g_prof.on = true;
    return WS_OK;
}

int ws_profile_reset(void) {
    g_prof.used = 0;
    return WS_OK;
}

int ws_profile_pause(int32_t paused) {
    g_prof.paused = paused != 0;
    return WS_OK;
}

int ws_profile_trace_dw(void* device_trace, int64_t tiles) {
    if (device_trace == nullptr) {
        g_dw_trace = nullptr;
        g_dw_trace_tiles = 0;
        return WS_OK;
    }
    if (tiles <= 0) return WS_ERR_SHAPE;
    if (!aligned(device_trace, 8)) return WS_ERR_ALIGN;
    g_dw_trace = static_cast<unsigned long long*>(device_trace);
    g_dw_trace_tiles = tiles;
    return WS_OK;
}

int32_t ws_profile_kernel_count(void) { return KID_COUNT; }

const char* ws_profile_kernel_name(int32_t kernel) {
    return (kernel >= 0 && kernel < KID_COUNT) ? kKernelNames[kernel] : "";
}

int ws_profile_read(int32_t kernel, double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return WS_ERR_NULL;
    if (kernel < 0 || kernel >= KID_COUNT) return WS_ERR_RANGE;
    double tot = 0.0;
    int64_t n = 0;
    for (int i = 0; i < g_prof.used; ++i) {
        if (g_prof.kid[i] != kernel) continue;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return WS_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return WS_ERR_HIP;
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *launches = n;
    return WS_OK;
}

}  // extern "C"
