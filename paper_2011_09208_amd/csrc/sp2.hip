// The other sharding pattern of the MatMul ShardingUnit (Section 3.2.2, "SP2"; compared with SP1 in
// Section 5.3.2): both inputs are cut along the CONTRACTION dimension, every device multiplies its
// feature slice by the matching slice of all class rows, and the full-width partial products are
// summed (an AllReduce in the paper).  What one device runs:
//   sp2_partial_logits   Z_s = X[:, D_s] . W[:, D_s]^T, all C classes, fp32 [B][C]
//   sp2_reduce_stats     z = sum_s Z_s + b;  per row: log-sum-exp, label logit, loss
// It exists to be measured against the class-split path: the partial logits it has to write and
// read back (S x B x C x 4 bytes) are the cost the class split avoids.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/whalesplit.h"
#include "gemm_core.h"

namespace ws {

struct Sp2Args {
    const uint16_t* X; int64_t ldx;      // [B][D_s]
    const uint16_t* W; int64_t ldw;      // [C][D_s]
    int B, Ds, C;
    int nBT, nCT;
    float* Z; int64_t ldz;               // [B][C] fp32
};

// Tile: M = batch rows (A = X slice), N = classes (B operand = W slice), both k-contiguous.  A lane
// holds 4 consecutive rows of one class column per accumulator, so the fp32 tile is written with
// 64-byte row segments per 16 lanes.
__global__ __launch_bounds__(NTHREADS) void sp2_partial_logits(Sp2Args a) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    const int tile = xcd_logical_tile(a.nBT * a.nCT);
    if (tile < 0) return;
    const int bt = tile % a.nBT, ct = tile / a.nBT;      // row tiles fastest: neighbours share the W panel
    acc_t acc;
    zero_acc(acc);
    const Operand A = make_operand(a.X, a.ldx, a.B, a.Ds);
    const Operand Bo = make_operand(a.W, a.ldw, a.C, a.Ds);
    gemm_mainloop<KC, KC>(acc, A, Bo, bt * TILE_M, ct * TILE_N, 0, a.Ds / TILE_K, lds);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int c = ct * TILE_N + wn * WAVE_N + 16 * nt + jl;
        if (c >= a.C) continue;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = bt * TILE_M + wm * WAVE_M + 16 * mt + 4 * g + v;
                if (row < a.B) __builtin_nontemporal_store(acc[mt][nt][v], a.Z + (int64_t)row * a.ldz + c);
            }
    }
}

constexpr int SP2_MAX_SLICES = 64;
struct Sp2Parts {
    const float* Z[SP2_MAX_SLICES];
    int64_t ldz[SP2_MAX_SLICES];
};

__device__ __forceinline__ void merge_pair(float& m, float& s, float m2, float s2) {
    const float M = fmaxf(m, m2);
    const float f1 = (m == -INFINITY) ? 0.0f : __expf(m - M);
    const float f2 = (m2 == -INFINITY) ? 0.0f : __expf(m2 - M);
    s = s * f1 + s2 * f2;
    m = M;
}

// One workgroup per row.  Thread t walks classes 4 t .. 4 t + 3, then 1024 further on, summing the S
// partial logits of each class in slice order (plus the bias) and folding the four values into its
// running (max, sum-exp); the 256 pairs are merged through LDS in a fixed order.
__global__ __launch_bounds__(256) void sp2_reduce_stats(Sp2Parts p, int S, const float* __restrict__ bias,
                                                        const int32_t* __restrict__ labels, int C,
                                                        float* __restrict__ logsumexp, float* __restrict__ loss_rows) {
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    __shared__ float sm[256], ss[256];
    const int row = blockIdx.x, tid = threadIdx.x;
    float m = -INFINITY, s = 0.0f;
    for (int c = 4 * tid; c < C; c += 1024) {
        if (c + 4 <= C) {
            f32x4 z = *reinterpret_cast<const f32x4*>(p.Z[0] + (int64_t)row * p.ldz[0] + c);
            for (int k = 1; k < S; ++k) z += *reinterpret_cast<const f32x4*>(p.Z[k] + (int64_t)row * p.ldz[k] + c);
            if (bias) z += *reinterpret_cast<const f32x4*>(bias + c);
            const float m4 = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
            const float s4 = __expf(z[0] - m4) + __expf(z[1] - m4) + __expf(z[2] - m4) + __expf(z[3] - m4);
            merge_pair(m, s, m4, s4);
        } else {
            for (int e = c; e < C; ++e) {
                float z = p.Z[0][(int64_t)row * p.ldz[0] + e];
                for (int k = 1; k < S; ++k) z += p.Z[k][(int64_t)row * p.ldz[k] + e];
                if (bias) z += bias[e];
                merge_pair(m, s, z, 1.0f);
            }
        }
    }
    sm[tid] = m;
    ss[tid] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) {
            merge_pair(m, s, sm[tid + w], ss[tid + w]);
            sm[tid] = m;
            ss[tid] = s;
        }
        __syncthreads();
    }
    if (tid == 0) {
        const float lse = m + __logf(s);
        const int y = labels[row];
        float t = 0.0f;
        if (y >= 0 && y < C) {
            t = p.Z[0][(int64_t)row * p.ldz[0] + y];
            for (int k = 1; k < S; ++k) t += p.Z[k][(int64_t)row * p.ldz[k] + y];
            if (bias) t += bias[y];
        }
        logsumexp[row] = lse;
        loss_rows[row] = lse - t;
    }
}

static inline bool al(const void* q, size_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) == 0; }

}  // namespace ws

using namespace ws;

extern "C" {

int ws_sp2_partial_logits(const void* X_slice, int64_t ldx, const void* W_slice, int64_t ldw, int32_t B,
                          int32_t D_slice, int32_t C, float* Z_partial, int64_t ldz, void* stream) {
    if (!X_slice || !W_slice || !Z_partial) return WS_ERR_NULL;
    if (B <= 0 || C <= 0 || D_slice <= 0 || D_slice % 64 != 0) return WS_ERR_SHAPE;
    if (ldx < D_slice || ldw < D_slice || ldz < C) return WS_ERR_SHAPE;
    // Z_partial: what ws_sp2_reduce_stats requires of its inputs, so a buffer accepted here is accepted there
    if (!al(Z_partial, 16) || ldz % 4) return WS_ERR_ALIGN;
    if (((int64_t)B + 256) * ldx * 2 >= ((int64_t)1 << 32) || ((int64_t)C + 256) * ldw * 2 >= ((int64_t)1 << 32))
        return WS_ERR_SHAPE;
    if (!al(X_slice, 16) || !al(W_slice, 16) || ldx % 8 || ldw % 8) return WS_ERR_ALIGN;
    Sp2Args a;
    a.X = static_cast<const uint16_t*>(X_slice); a.ldx = ldx;
    a.W = static_cast<const uint16_t*>(W_slice); a.ldw = ldw;
    a.B = B; a.Ds = D_slice; a.C = C;
    a.nBT = (B + 255) / 256; a.nCT = (C + 255) / 256;
    a.Z = Z_partial; a.ldz = ldz;
    const int tiles = a.nBT * a.nCT;
    hipLaunchKernelGGL(sp2_partial_logits, dim3(8 * ((tiles + 7) / 8)), dim3(NTHREADS), 0,
                       static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

int ws_sp2_reduce_stats(const float* const* Z_partials, const int64_t* ldz, int32_t S, const float* bias,
                        const int32_t* labels, int32_t B, int32_t C, float* logsumexp, float* loss_rows,
                        void* stream) {
    if (!Z_partials || !ldz || !labels || !logsumexp || !loss_rows) return WS_ERR_NULL;
    if (S < 1 || S > SP2_MAX_SLICES) return WS_ERR_RANGE;
    if (B <= 0 || C <= 0) return WS_ERR_SHAPE;
    Sp2Parts p;
    for (int k = 0; k < SP2_MAX_SLICES; ++k) {
        if (k >= S) {
            p.Z[k] = nullptr; p.ldz[k] = 0;
            continue;
        }
        if (!Z_partials[k]) return WS_ERR_NULL;
        if (ldz[k] < C) return WS_ERR_SHAPE;
        if (!al(Z_partials[k], 16) || ldz[k] % 4) return WS_ERR_ALIGN;
        p.Z[k] = Z_partials[k]; p.ldz[k] = ldz[k];
    }
    if ((bias && !al(bias, 16)) || !al(labels, 4) || !al(logsumexp, 4) || !al(loss_rows, 4)) return WS_ERR_ALIGN;
    hipLaunchKernelGGL(sp2_reduce_stats, dim3(B), dim3(256), 0, static_cast<hipStream_t>(stream), p, S, bias, labels,
                       C, logsumexp, loss_rows);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

}  // extern "C"
