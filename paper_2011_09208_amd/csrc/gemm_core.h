// Shared bf16 MFMA GEMM main loop for gfx950 (MI355X), used by all four contractions
// of the split fully-connected head.
//
// One workgroup of 512 threads (8 wave64s, two per SIMD) owns a 256 x 256 output tile
// and walks the contraction in steps of 64.  The waves form a 2 (M) x 4 (N) grid; each
// owns a 128 x 64 sub-tile held as 8 x 4 accumulators of v_mfma_f32_16x16x32_bf16 (measured
// about 7 % faster than the 32x32x16 form under the chip's power limit: it moves half as many
// accumulator registers per flop).
//
// An operand tile is staged in LDS in one of two layouts, chosen by how the operand
// lies in memory relative to the contraction index k:
//   KC ("k contiguous"): memory is [row][k]; LDS holds [256 rows][64 k] (128 B per row,
//       16-byte chunks XOR-swizzled by (row >> 1) & 7); a lane's MFMA fragment (8
//       consecutive k of one row) is one ds_read_b128.
//   KS ("k strided"):    memory is [k][col]; LDS holds [64 k][256 cols] (512 B per k-row,
//       16-byte chunks XOR-swizzled by ((k >> 3) & 3) << 1 | (k & 3) << 3); the fragment is
//       gathered with two ds_read_b64_tr_b16 transpose reads (4 consecutive k of one column each).
// Lane layouts used (checked on the hardware): for v_mfma_f32_16x16x32_bf16 lane l
// supplies row l % 16, k = 8 * (l / 16) .. + 7 of either operand; accumulator register v
// of lane l is element (4 * (l / 16) + v, l % 16).  ds_read_b64_tr_b16
// works on blocks of 16 lanes: lane i of a block receives, as element e, the (i % 4)-th
// 16-bit value of the 8 bytes addressed by lane 4 * e + i / 4 of the same block.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ws {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int TILE_M = 256;
constexpr int TILE_N = 256;
constexpr int TILE_K = 64;
constexpr int NTHREADS = 512;
constexpr int WAVE_M = 128;     // rows of the output tile one wave owns
constexpr int WAVE_N = 64;
constexpr int MT = WAVE_M / 16; // 16 x 16 MFMA tiles per wave along M: 8
constexpr int NT = WAVE_N / 16; // and along N: 4
constexpr int OPERAND_TILE_BYTES = 256 * TILE_K * 2;           // 32 KiB
constexpr int STAGE_BYTES = 2 * OPERAND_TILE_BYTES;            // A + B
constexpr int LDS_BYTES = 2 * STAGE_BYTES;                     // double buffered: 128 KiB

enum { KC = 0, KS = 1 };

// One GEMM operand in global memory (16-bit elements), addressed through a buffer resource:
//   KC: element (row, k) at base[row * ld + k];   KS: element (k, col) at base[k * ld + col].
// Loads are buffer_load_dwordx4 with a scalar resource, a scalar offset (the k-step and the tile
// quarter) and ONE 32-bit per-lane offset per operand that never changes inside the main loop.
// The resource covers exactly rows x cols of the matrix: a tile may hang over its end (ragged row or
// class counts, the last k-step of a contraction) and the overhang reads as zeros, as the hardware
// bounds check returns 0 beyond the resource.  Offsets are 32-bit: (rows + 256) * ld * 2 bytes must stay
// below 4 GiB (checked on the host).
struct Operand {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t ld;        // row pitch in elements
};

// `rows` x `cols` elements are valid (KC: rows x k extent; KS: k extent x columns).
__device__ __forceinline__ Operand make_operand(const uint16_t* base, int64_t ld, int64_t rows, int64_t cols) {
    const int64_t bytes = ((rows - 1) * ld + cols) * 2;
    Operand op;
    op.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, (int)(uint32_t)bytes, 0x00020000);
    op.ld = (uint32_t)ld;
    return op;
}

// ---- global -> registers -> LDS staging ---------------------------------------------------
// A 32 KiB operand tile is 2048 chunks of 16 bytes; thread t moves chunks t, t + 512, t + 1024 and
// t + 1536.  Chunk set j (one chunk per thread) is "quarter j" of the tile: rows 64 j .. 64 j + 63 of
// a KC tile, k-rows 16 j .. 16 j + 15 of a KS tile.

// Chunk swizzle of a KS tile.  A transposing read is served half a wave at a time; the 32 lanes of a
// half cover 4 k-rows (k & 3) in each of 2 lane blocks 8 k-rows apart ((k >> 3) & 1), two adjacent
// chunks and both 8-byte halves of a chunk each.  Those 16 (k-row, chunk) pairs must fall into 16
// different chunks modulo 16 (256 bytes span all banks): k & 3 goes to chunk bits 2-3, (k >> 3) & 1 to
// bit 1, the two adjacent chunks differ in bit 0.  Bit 4 of k only separates the two halves of the wave.
// Bits 2 and 5 of k are left out so that the reads 4 and 32 k-rows further on keep the same pattern.
__device__ __forceinline__ int ks_swizzle(int k) {
    return (((k >> 3) & 1) << 1) | ((k & 3) << 2) | (((k >> 4) & 1) << 4);
}

// Per-lane byte offset of a thread's chunk in quarter 0 of the tile whose first row (KC) or first
// column (KS) is o0, at k = 0.
template <int KIND>
__device__ __forceinline__ uint32_t tile_lane_offset(const Operand& op, int o0, int tid) {
    if (KIND == KC) return ((uint32_t)(o0 + (tid >> 3)) * op.ld + (uint32_t)((tid & 7) * 8)) * 2u;
    return ((uint32_t)(tid >> 5) * op.ld + (uint32_t)(o0 + (tid & 31) * 8)) * 2u;
}

// Loads this thread's chunk of quarter j of the tile at contraction offset k0.
template <int KIND>
__device__ __forceinline__ u32x4 quarter_g2r(const Operand& op, uint32_t lane_off, int k0, int j) {
    const uint32_t soff = KIND == KC ? ((uint32_t)k0 + (uint32_t)(64 * j) * op.ld) * 2u
                                     : ((uint32_t)(k0 + 16 * j) * op.ld) * 2u;
    return __builtin_amdgcn_raw_buffer_load_b128(op.rsrc, (int)lane_off, (int)soff, 0);
}

template <int KIND>
__device__ __forceinline__ void quarter_r2s(char* lds, const u32x4& v, int tid, int j) {
    const int q = tid + NTHREADS * j;
    int off;
    if (KIND == KC) {
        const int row = q >> 3, ch = q & 7;
        off = row * 128 + ((ch ^ ((row >> 1) & 7)) << 4);
    } else {
        const int kr = q >> 5, ch = q & 31;
        off = kr * 512 + ((ch ^ ks_swizzle(kr)) << 4);
    }
    *reinterpret_cast<u32x4*>(lds + off) = v;
}

// ---- LDS -> MFMA fragments ------------------------------------------------------------------

// Per-lane byte offsets into an operand tile, computed once per kernel.
template <int KIND, int NTILES>
struct FragAddr {
    int off[KIND == KC ? 2 : NTILES];   // KC: one per 32-wide k-substep; KS: one per 16-wide tile

    // `w0` = first row/column of this wave's sub-tile inside the 256-wide operand tile.
    __device__ __forceinline__ void init(int lane, int w0) {
        const int i = lane & 15, g = lane >> 4;
        if (KIND == KC) {
            const int sw = (i >> 1) & 7;            // w0 and 16 * t are multiples of 16: no effect on the swizzle
#pragma unroll
            for (int s = 0; s < 2; ++s) off[s] = (w0 + i) * 128 + (((4 * s + g) ^ sw) << 4);
        } else {
            const int x = i >> 2;                    // k-row within the group of four == (k & 3)
            const int krow = 8 * g + x;              // substeps add multiples of 32, the second read 4
#pragma unroll
            for (int t = 0; t < NTILES; ++t) {
                const int col = w0 + 16 * t + 4 * (i & 3);
                off[t] = krow * 512 + (((col >> 3) ^ ks_swizzle(krow)) << 4) + ((col & 7) << 1);
            }
        }
    }

    // Fragment of 16-wide tile t for k-substep s (32 k each) from the operand tile at `lds`.
    __device__ __forceinline__ bf16x8 load(const char* lds, int t, int s) const {
        if (KIND == KC) {
            return *reinterpret_cast<const bf16x8*>(lds + off[s] + t * (16 * 128));
        } else {
            typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
            const char* p = lds + off[t] + s * (32 * 512);
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * 512));
            s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    }
};

// ---- main loop ---------------------------------------------------------------------------------

// Scheduling hint for one slot of the software pipeline: N MFMAs; NR LDS reads go with the first
// MFMAs (so that they land before the slot ends), then NW LDS writes, then NV global loads with the
// last MFMAs.  The instructions are written before the hint; the hint only fixes their interleaving
// (LDS reads stay ahead of LDS writes, as the compiler must assume they may alias).
template <int I, int N, int NR, int NW, int NV>
struct SlotSched {
    static __device__ __forceinline__ void apply() {
        constexpr int H = (N + 1) / 2 + 1;
        constexpr int r = I < H ? (NR * (I + 1) + H - 1) / H - (NR * I + H - 1) / H : 0;
        constexpr int w = (I >= N - 1 - NW && I < N - 1) ? 1 : 0;
        constexpr int v = (I >= N - NV) ? 1 : 0;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
        if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);   // LDS reads
        if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);   // LDS writes
        if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);   // global loads
        if constexpr (I + 1 < N) SlotSched<I + 1, N, NR, NW, NV>::apply();
        else __builtin_amdgcn_sched_barrier(0);      // nothing moves across the end of a slot
    }
};

// acc[mt][nt] += A(m0 .. m0+255, k) * B(n0 .. n0+255, k) for k in [k_begin, k_begin + 64 * k_steps).
// For a KC operand o0 is its first row; for a KS operand its first column.
// Ends with a workgroup barrier, so LDS may be reused by the caller right away.
//
// Software pipeline.  LDS holds two stages (k-step j in stage j & 1).  Iteration j multiplies
// k-step j in four slots of 16 MFMAs each: (k-substep 0 | 1 of 32) x (upper | lower 64 rows of the
// wave's sub-tile); the fragments of a slot are read from LDS one slot ahead (A fragments every slot,
// B fragments every other slot).  The tiles are staged through registers one quarter at a time,
// so that LDS writes and global loads are spread evenly over the iteration and every global load
// has a full iteration to land:
//   slot x = 0, 1, 2:  quarter x of k-step j + 1: registers -> stage (j + 1) & 1; then the same
//                      registers <- quarter x of k-step j + 2 from global memory
//   barrier            (every wave has finished reading stage j & 1 and writing stage (j + 1) & 1)
//   slot 3:            quarter 3 of k-step j + 2: registers -> stage j & 1 (free now); then the
//                      registers <- quarter 3 of k-step j + 3
// k-steps beyond the last are clamped to the last one (a harmless reload).  Rows, columns or k beyond
// an operand's extent read as zeros.
typedef f32x4 acc_t[MT][NT];

// `descending` (uniform over the workgroup): walk the k-steps from the last to the first.  Tiles that follow each
// other on a compute unit and share an operand panel can alternate the direction, so that the second finds
// the end of the panel, which the first has just read, still in the L2.
template <int AKIND, int BKIND>
__device__ __forceinline__ void gemm_mainloop(acc_t& acc, const Operand& A, const Operand& Bop,
                                              int m0, int n0, int k_begin, int k_steps, char* lds,
                                              bool descending = false) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    constexpr int HM = MT / 2;                                   // M tiles per slot
    constexpr int RA = HM * (AKIND == KC ? 1 : 2);               // LDS reads for a slot's A fragments
    constexpr int RB = NT * (BKIND == KC ? 1 : 2);               // and for a substep's B fragments
    constexpr int NMFMA = HM * NT;
    const int last = k_steps - 1;

    FragAddr<AKIND, MT> fa;
    FragAddr<BKIND, NT> fb;
    fa.init(lane, wm * WAVE_M);
    fb.init(lane, wn * WAVE_N);

    u32x4 sa[4], sb[4];
    bf16x8 af[2][HM], bfr[2][NT];

    auto load_a = [&](int set, const char* la, int s, int half) {
#pragma unroll
        for (int t = 0; t < HM; ++t) af[set][t] = fa.load(la, HM * half + t, s);
    };
    auto load_b = [&](int set, const char* la, int s) {
#pragma unroll
        for (int t = 0; t < NT; ++t) bfr[set][t] = fb.load(la + OPERAND_TILE_BYTES, t, s);
    };
    auto mfmas = [&](int aset, int bset, int half) {
#pragma unroll
        for (int i = 0; i < HM; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[HM * half + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[aset][i], bfr[bset][j],
                                                                                acc[HM * half + i][j], 0, 0, 0);
    };
    const int k_first = descending ? k_begin + last * TILE_K : k_begin;
    const int k_stride = descending ? -TILE_K : TILE_K;
    auto kofs = [&](int step) { return k_first + (step < last ? step : last) * k_stride; };
    const uint32_t a_off = tile_lane_offset<AKIND>(A, m0, tid);
    const uint32_t b_off = tile_lane_offset<BKIND>(Bop, n0, tid);
    auto g2r = [&](int quarter, int step) {
        sa[quarter] = quarter_g2r<AKIND>(A, a_off, kofs(step), quarter);
        sb[quarter] = quarter_g2r<BKIND>(Bop, b_off, kofs(step), quarter);
    };
    auto r2s = [&](int quarter, char* stage) {
        quarter_r2s<AKIND>(stage, sa[quarter], tid, quarter);
        quarter_r2s<BKIND>(stage + OPERAND_TILE_BYTES, sb[quarter], tid, quarter);
    };

    // prologue: stage 0 <- k-step 0; quarter 3 of k-step 1 -> stage 1; registers <- what the loop expects.
    // Quarter 3 of k-step 1 is fetched together with k-step 0 (into spare registers), so the fill costs
    // one global-memory latency, not two.
#pragma unroll
    for (int q = 0; q < 4; ++q) g2r(q, 0);
    const u32x4 a31 = quarter_g2r<AKIND>(A, a_off, kofs(1), 3);
    const u32x4 b31 = quarter_g2r<BKIND>(Bop, b_off, kofs(1), 3);
#pragma unroll
    for (int q = 0; q < 4; ++q) r2s(q, lds);
    quarter_r2s<AKIND>(lds + STAGE_BYTES, a31, tid, 3);
    quarter_r2s<BKIND>(lds + STAGE_BYTES + OPERAND_TILE_BYTES, b31, tid, 3);
#pragma unroll
    for (int q = 0; q < 3; ++q) g2r(q, 1);
    g2r(3, 2);
    __syncthreads();
    load_a(0, lds, 0, 0);
    load_b(0, lds, 0);

    for (int j = 0; j < last; ++j) {
        char* lc = lds + (j & 1) * STAGE_BYTES;          // stage of k-step j
        char* ln = lds + ((j + 1) & 1) * STAGE_BYTES;    // stage of k-step j + 1
        // slot 0: substep 0, upper rows
        load_a(1, lc, 0, 1);
        mfmas(0, 0, 0);
        r2s(0, ln);
        g2r(0, j + 2);
        SlotSched<0, NMFMA, RA, 2, 2>::apply();
        // slot 1: substep 0, lower rows
        load_a(0, lc, 1, 0);
        load_b(1, lc, 1);
        mfmas(1, 0, 1);
        r2s(1, ln);
        g2r(1, j + 2);
        SlotSched<0, NMFMA, RA + RB, 2, 2>::apply();
        // slot 2: substep 1, upper rows
        load_a(1, lc, 1, 1);
        mfmas(0, 1, 0);
        r2s(2, ln);
        g2r(2, j + 2);
        SlotSched<0, NMFMA, RA, 2, 2>::apply();
        __syncthreads();
        // slot 3: substep 1, lower rows
        load_a(0, ln, 0, 0);
        load_b(0, ln, 0);
        mfmas(1, 1, 1);
        r2s(3, lc);
        g2r(3, j + 3);
        SlotSched<0, NMFMA, RA + RB, 2, 2>::apply();
    }
    {   // last k-step: nothing left to stage
        const char* lc = lds + (last & 1) * STAGE_BYTES;
        load_a(1, lc, 0, 1);
        mfmas(0, 0, 0);
        SlotSched<0, NMFMA, RA, 0, 0>::apply();
        load_a(0, lc, 1, 0);
        load_b(1, lc, 1);
        mfmas(1, 0, 1);
        SlotSched<0, NMFMA, RA + RB, 0, 0>::apply();
        load_a(1, lc, 1, 1);
        mfmas(0, 1, 0);
        SlotSched<0, NMFMA, RA, 0, 0>::apply();
        mfmas(1, 1, 1);
    }
    __syncthreads();
}

__device__ __forceinline__ void zero_acc(acc_t& acc) {
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;
}

// ---- thin tiles ------------------------------------------------------------------------------------
// A launch whose tile count is not a multiple of the 256 compute units ends with a round in which
// most of them idle.  The tiles of that last round can instead be cut into four "thin" tiles of
// 256 x 64 (one wave column of a full tile each) and handed to four times as many workgroups.  A thin
// tile does a quarter of the MFMA work for 5/8 of the staging traffic, so it runs at the pace of its
// LDS writes, about a quarter to a third of a full tile's time.  Both operands are KC.
constexpr int THIN_N = WAVE_N;                         // 64 columns
constexpr int THIN_WAVE_M = TILE_M / 8;                // a wave of a thin tile: 32 rows x 64 columns
constexpr int THIN_MT = THIN_WAVE_M / 16, THIN_NT = THIN_N / 16;
constexpr int THIN_STAGE_BYTES = OPERAND_TILE_BYTES + THIN_N * TILE_K * 2;    // 32 KiB A + 8 KiB B
typedef f32x4 thin_acc_t[THIN_MT][THIN_NT];

// A thin tile's B operand may also be k-strided (memory [k][col]): LDS then holds [64 k][64 cols], 128 bytes per
// k-row, 16-byte chunks XOR-ed with thin_ks_swizzle(k).  A transposing read is served half a wave at a time:
// 8 k-rows (k & 3 and bit 3 of k), two adjacent chunks and both halves of a chunk; k & 1 picks the 128-byte
// half of the bank window, bits 1 and 3 of k go to chunk bits 1-2, the adjacent chunks differ in bit 0.
__device__ __forceinline__ int thin_ks_swizzle(int k) { return (((k >> 1) & 1) << 1) | (((k >> 3) & 1) << 2); }

// Byte offset of a thread's chunk of the k-strided thin B tile whose first column is n0, at k = 0: thread t
// moves chunk t % 8 of k-row t / 8.
__device__ __forceinline__ uint32_t thin_ks_lane_offset(const Operand& op, int n0, int tid) {
    return ((uint32_t)(tid >> 3) * op.ld + (uint32_t)(n0 + (tid & 7) * 8)) * 2u;
}
__device__ __forceinline__ u32x4 thin_ks_g2r(const Operand& op, uint32_t lane_off, int k0) {
    return __builtin_amdgcn_raw_buffer_load_b128(op.rsrc, (int)lane_off, (int)((uint32_t)k0 * op.ld * 2u), 0);
}
__device__ __forceinline__ void thin_ks_r2s(char* lds, const u32x4& v, int tid) {
    const int kr = tid >> 3, ch = tid & 7;
    *reinterpret_cast<u32x4*>(lds + kr * 128 + ((ch ^ thin_ks_swizzle(kr)) << 4)) = v;
}
struct ThinKsFrag {
    int off[THIN_N / 16];
    __device__ __forceinline__ void init(int lane) {
        const int i = lane & 15, g = lane >> 4;
        const int krow = 8 * g + (i >> 2);
#pragma unroll
        for (int t = 0; t < THIN_N / 16; ++t) {
            const int col = 16 * t + 4 * (i & 3);
            off[t] = krow * 128 + (((col >> 3) ^ thin_ks_swizzle(krow)) << 4) + ((col & 7) << 1);
        }
    }
    __device__ __forceinline__ bf16x8 load(const char* lds, int t, int s) const {
        typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
        const char* p = lds + off[t] + s * (32 * 128);
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * 128));
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
};

// acc[mt][nt] += A(m0 .. m0+255, k) * B(n0 .. n0+63, k) for k in [k_begin, k_begin + 64 * k_steps);
// wave w holds rows 32 w .. 32 w + 31.  BKIND KS: B is k-strided, n0 its first column.  Two LDS stages, the same software pipeline as the full tile in
// two slots of 8 MFMAs per k-step: slot A multiplies k-substep 0 while the fragments of substep 1 are
// read, the next k-step goes registers -> LDS and the one after it global -> registers; after the
// barrier slot B multiplies substep 1 while the first fragments of the next k-step are read.
// k-steps beyond the last are clamped to the last one (a harmless reload).  Ends with a workgroup barrier.
template <int BKIND = KC>
__device__ __forceinline__ void thin_mainloop(thin_acc_t& acc, const Operand& A, const Operand& Bop, int m0, int n0,
                                              int k_begin, int k_steps, char* lds, bool descending = false) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    FragAddr<KC, THIN_MT> fa;
    FragAddr<KC, THIN_NT> fb;
    ThinKsFrag fbs;
    fa.init(lane, wave * THIN_WAVE_M);
    if (BKIND == KC) fb.init(lane, 0);
    else fbs.init(lane);
    const uint32_t a_off = tile_lane_offset<KC>(A, m0, tid);
    // KC: thread t moves chunk t % 8 of row t / 8 of the 64; KS: chunk t % 8 of k-row t / 8
    const uint32_t b_off = BKIND == KC ? tile_lane_offset<KC>(Bop, n0, tid) : thin_ks_lane_offset(Bop, n0, tid);
    const int last = k_steps - 1;
    const int k_first = descending ? k_begin + last * TILE_K : k_begin;
    const int k_stride = descending ? -TILE_K : TILE_K;
    constexpr int NM = THIN_MT * THIN_NT, NR = THIN_MT + THIN_NT * (BKIND == KC ? 1 : 2);
    u32x4 ra[4], rb;
    bf16x8 af[2][THIN_MT], bfr[2][THIN_NT];
    auto g2r = [&](int step) {
        const int k0 = k_first + (step < last ? step : last) * k_stride;
#pragma unroll
        for (int q = 0; q < 4; ++q) ra[q] = quarter_g2r<KC>(A, a_off, k0, q);
        rb = BKIND == KC ? quarter_g2r<KC>(Bop, b_off, k0, 0) : thin_ks_g2r(Bop, b_off, k0);
    };
    auto r2s = [&](char* stage) {
#pragma unroll
        for (int q = 0; q < 4; ++q) quarter_r2s<KC>(stage, ra[q], tid, q);
        if (BKIND == KC) quarter_r2s<KC>(stage + OPERAND_TILE_BYTES, rb, tid, 0);
        else thin_ks_r2s(stage + OPERAND_TILE_BYTES, rb, tid);
    };
    auto frags = [&](int set, const char* stage, int s) {
#pragma unroll
        for (int i = 0; i < THIN_MT; ++i) af[set][i] = fa.load(stage, i, s);
#pragma unroll
        for (int i = 0; i < THIN_NT; ++i)
            bfr[set][i] = BKIND == KC ? fb.load(stage + OPERAND_TILE_BYTES, i, s) : fbs.load(stage + OPERAND_TILE_BYTES, i, s);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int i = 0; i < THIN_MT; ++i)
#pragma unroll
            for (int jn = 0; jn < THIN_NT; ++jn)
                acc[i][jn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[set][i], bfr[set][jn], acc[i][jn], 0, 0, 0);
    };
    g2r(0);
    r2s(lds);
    g2r(1);
    __syncthreads();
    frags(0, lds, 0);
    for (int j = 0; j < last; ++j) {
        const char* cur = lds + (j & 1) * THIN_STAGE_BYTES;
        char* nxt = lds + ((j + 1) & 1) * THIN_STAGE_BYTES;
        frags(1, cur, 1);
        mfmas(0);
        r2s(nxt);                  // free since the barrier of the iteration before
        g2r(j + 2);
        SlotSched<0, NM, NR, 5, 5>::apply();
        __syncthreads();
        frags(0, nxt, 0);
        mfmas(1);
        SlotSched<0, NM, NR, 0, 0>::apply();
    }
    {
        const char* cur = lds + (last & 1) * THIN_STAGE_BYTES;
        frags(1, cur, 1);
        mfmas(0);
        SlotSched<0, NM, NR, 0, 0>::apply();
        mfmas(1);
    }
    __syncthreads();
}

// How a launch of n_tiles full tiles is cut: the tiles of the last, partial round become thin tiles
// when that round would leave at least half of the compute units idle.
struct TilePlan {
    int n_full;      // full tiles, logical ids 0 .. n_full - 1 (workgroups 0 .. 8 * ceil(n_full / 8) - 1)
    int n_thin;      // thin tiles: 4 per remaining full tile, workgroups thin_first .. thin_first + n_thin - 1
    int thin_first;
};

// Workgroups are handed to the 8 XCDs round-robin by their linear id; each XCD has its own L2.
// Map the hardware id to a logical tile id so that each XCD walks one contiguous range of
// logical tiles (tiles that share an operand panel are numbered next to each other).
// The grid must hold 8 * ceil(n_tiles / 8) workgroups; returns -1 for the surplus ones.
__device__ __forceinline__ int xcd_logical_tile(int n_tiles) {
    const int per = (n_tiles + 7) >> 3;
    const int bid = blockIdx.x;
    const int t = (bid & 7) * per + (bid >> 3);
    return t < n_tiles ? t : -1;
}

// Round-to-nearest-even conversion of two floats to a packed bf16 pair.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 r = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// ---- output tiles through LDS ------------------------------------------------------------------------
// The MFMA accumulator layout gives a lane one N index and groups of four consecutive M indices, which
// makes direct global stores 8 or 16 bytes wide and scattered over 16 rows.  Instead the 256 x 256 tile
// is rounded to bf16 and laid out in LDS as [n][m] (512 bytes per n; it fills the 128 KiB the main loop
// no longer needs), then written out row by row.  Every n-row starts at bank 0, so the eight-byte slots of
// a row are XOR-ed with n & 15.  Measured on gfx950 with the bank-conflict counter:
//   accumulator writes (ds_write_b64): served 16 consecutive lanes at a time, and the 16 slots must differ
//       modulo 16 (a 128-byte window).  The 16 lanes are 16 consecutive n and one slot s, and s ^ (n & 15)
//       takes every value modulo 16 once;
//   row reads (ds_read_b128): served in the lane sets {0-3, 12-15, 20-27} and {4-11, 16-19, 28-31} of each
//       half wave, whose 16-byte chunks must differ modulo 16 (a 256-byte window).  A lane's chunk is two
//       adjacent slots, swapped when n is odd; both lane sets cover every chunk index modulo 16 once and
//       c -> c ^ ((n & 15) >> 1) permutes them.

__device__ __forceinline__ int out_tile_swizzle(int n) { return n & 15; }

// Byte offset of element (n, m) in the swizzled tile; m must be a multiple of 4 for 8-byte accesses.
__device__ __forceinline__ int out_tile_offset(int n, int m) {
    return n * 512 + (((m >> 2) ^ out_tile_swizzle(n)) << 3) + ((m & 3) << 1);
}

__device__ __forceinline__ void acc_to_lds_bf16(const acc_t& acc, char* lds) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3, g = lane >> 4, jl = lane & 15;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = wn * WAVE_N + 16 * nt + jl;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            u32x2 p;
            p[0] = pack_bf16(acc[mt][nt][0], acc[mt][nt][1]);
            p[1] = pack_bf16(acc[mt][nt][2], acc[mt][nt][3]);
            *reinterpret_cast<u32x2*>(lds + out_tile_offset(n, wm * WAVE_M + 16 * mt + 4 * g)) = p;
        }
    }
}

// Writes the LDS tile to out[n][m] (row pitch ld elements, `out` = address of element (0, 0) of the
// tile), rows n < n_valid and columns m < m_valid only.  A wave stores two whole 512-byte rows per
// instruction; a chunk that m_valid cuts (m_valid not a multiple of 8) goes out element by element.
__device__ __forceinline__ void lds_tile_store_rows(const char* lds, uint16_t* out, int64_t ld, int n_valid,
                                                    int m_valid) {
    const int tid = threadIdx.x;
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int q = tid + NTHREADS * i;
        const int n = q >> 5, cq = q & 31;
        if (n < n_valid && cq * 8 < m_valid) {
            // the two 8-byte halves of a 16-byte chunk stay in one chunk, swapped when the swizzle is odd
            const int g = out_tile_swizzle(n);
            u32x4 v = *reinterpret_cast<const u32x4*>(lds + n * 512 + ((cq ^ (g >> 1)) << 4));
            if (g & 1) v = __builtin_shufflevector(v, v, 2, 3, 0, 1);
            uint16_t* o = out + (int64_t)n * ld + cq * 8;
            if (cq * 8 + 8 <= m_valid) {
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(o));
            } else {
                const int left = m_valid - cq * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < left) o[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

// The LDS tile holds a gradient; out[n][m] <- bf16(out[n][m] - lr * tile[n][m]) for the same rows and
// columns as lds_tile_store_rows, each 16-byte chunk read, updated in fp32 and written back.
__device__ __forceinline__ void lds_tile_update_rows(const char* lds, uint16_t* out, int64_t ld, int n_valid,
                                                     int m_valid, float lr) {
    const int tid = threadIdx.x;
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int q = tid + NTHREADS * i;
        const int n = q >> 5, cq = q & 31;
        if (n < n_valid && cq * 8 < m_valid) {
            const int g = out_tile_swizzle(n);
            u32x4 gr = *reinterpret_cast<const u32x4*>(lds + n * 512 + ((cq ^ (g >> 1)) << 4));
            if (g & 1) gr = __builtin_shufflevector(gr, gr, 2, 3, 0, 1);
            uint16_t* o = out + (int64_t)n * ld + cq * 8;
            if (cq * 8 + 8 <= m_valid) {
                const u32x4 w = *reinterpret_cast<const u32x4*>(o);
                u32x4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float w0 = __uint_as_float(w[e] << 16), w1 = __uint_as_float(w[e] & 0xffff0000u);
                    const float g0 = __uint_as_float(gr[e] << 16), g1 = __uint_as_float(gr[e] & 0xffff0000u);
                    r[e] = pack_bf16(fmaf(-lr, g0, w0), fmaf(-lr, g1, w1));
                }
                *reinterpret_cast<u32x4*>(o) = r;
            } else {
                const int left = m_valid - cq * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < left) {
                        const float wv = __uint_as_float((uint32_t)o[e] << 16);
                        const float gv = __uint_as_float((uint32_t)(uint16_t)(gr[e >> 1] >> (16 * (e & 1))) << 16);
                        o[e] = (uint16_t)(pack_bf16(fmaf(-lr, gv, wv), 0.0f) & 0xffffu);
                    }
            }
        }
    }
}

}  // namespace ws
