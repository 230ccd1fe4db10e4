// Diagnostic kernels that measure what the machine allows the GEMM main loop of this library, so that the
// figures the split-FC kernels reach can be read against a measured ceiling and not only the nominal peak:
//   ws_probe_mfma_loop   nothing but v_mfma_f32_16x16x32_bf16 on operands that sit in registers
//   ws_probe_gemm        the shared main loop (gemm_core.h) alone as a plain C = A . B^T, bf16 out
// The matrix cores of this part run into a power limit that depends on the operand data, so both take
// the operand values from the caller (constant or random).  Not part of the paper's method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/whalesplit.h"
#include "gemm_core.h"

namespace ws {

// Every wave keeps 8 A and 8 B fragments (read once from `frags`, [16][512] fragments of 16 bytes) and 16
// accumulators; one round is 128 MFMAs (every A fragment pair against every B fragment).
__global__ __launch_bounds__(NTHREADS) void probe_mfma_loop(const u32x4* __restrict__ frags, int rounds,
                                                             float* __restrict__ sink) {
    const int t = threadIdx.x;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, frags[i * NTHREADS + t]);
        b[i] = __builtin_bit_cast(bf16x8, frags[(i + 8) * NTHREADS + t]);
    }
    f32x4 acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int o = 0; o < 8; ++o)
#pragma unroll
            for (int j = 0; j < 16; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j & 7], b[(j + o) & 7], acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    sink[blockIdx.x * NTHREADS + t] = s;
}

struct ProbeGemmArgs {
    const uint16_t* A; int64_t lda;
    const uint16_t* B; int64_t ldb;
    uint16_t* C; int64_t ldc;
    int M, N, K, nMT, nNT;
};

// C[n][m] = sum_k A[m][k] * B[n][k]: both operands k-contiguous, output through LDS in whole rows, as the
// dW kernel writes its tiles.
__global__ __launch_bounds__(NTHREADS) void probe_gemm(ProbeGemmArgs p) {
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    const int tile = xcd_logical_tile(p.nMT * p.nNT);
    if (tile < 0) return;
    const int mt = tile % p.nMT, nt = tile / p.nMT;
    acc_t acc;
    zero_acc(acc);
    const Operand A = make_operand(p.A, p.lda, p.M, p.K);
    const Operand Bo = make_operand(p.B, p.ldb, p.N, p.K);
    gemm_mainloop<KC, KC>(acc, A, Bo, mt * TILE_M, nt * TILE_N, 0, p.K / TILE_K, lds);
    acc_to_lds_bf16(acc, lds);
    __syncthreads();
    lds_tile_store_rows(lds, p.C + (int64_t)nt * TILE_N * p.ldc + mt * TILE_M, p.ldc, TILE_N, TILE_M);
}

static inline bool al16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }

}  // namespace ws

using namespace ws;

extern "C" {

int ws_probe_mfma_loop(const void* fragments, int32_t rounds, int32_t workgroups, float* sink, void* stream) {
    if (!fragments || !sink) return WS_ERR_NULL;
    if (rounds <= 0 || workgroups <= 0 || workgroups > 65536) return WS_ERR_RANGE;
    if (!al16(fragments) || !al16(sink)) return WS_ERR_ALIGN;
    hipLaunchKernelGGL(probe_mfma_loop, dim3(workgroups), dim3(NTHREADS), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(fragments), rounds, sink);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

int ws_probe_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, int32_t M, int32_t N, int32_t K,
                  void* C, int64_t ldc, void* stream) {
    if (!A || !B || !C) return WS_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || M % 256 || N % 256 || K % 64) return WS_ERR_SHAPE;
    if (lda < K || ldb < K || ldc < M) return WS_ERR_SHAPE;
    if (((int64_t)M + 256) * lda * 2 >= ((int64_t)1 << 32) || ((int64_t)N + 256) * ldb * 2 >= ((int64_t)1 << 32))
        return WS_ERR_SHAPE;
    if (!al16(A) || !al16(B) || !al16(C) || lda % 8 || ldb % 8 || ldc % 8) return WS_ERR_ALIGN;
    ProbeGemmArgs p;
    p.A = static_cast<const uint16_t*>(A); p.lda = lda;
    p.B = static_cast<const uint16_t*>(B); p.ldb = ldb;
    p.C = static_cast<uint16_t*>(C); p.ldc = ldc;
    p.M = M; p.N = N; p.K = K; p.nMT = M / 256; p.nNT = N / 256;
    const int tiles = p.nMT * p.nNT;
    hipLaunchKernelGGL(probe_gemm, dim3(8 * ((tiles + 7) / 8)), dim3(NTHREADS), 0, static_cast<hipStream_t>(stream), p);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

}  // extern "C"
