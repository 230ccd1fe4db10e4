// The two ends of the bridge layer (Section 3.2.3) as they look on one device:
//   bridge_gather            concatenation of the parts other devices produced, along the batch
//                            dimension (replicate pattern) or the split dimension (split pattern)
//   bridge_reduce_partition  the way back in front of a split TaskGraph: the shards' partial
//                            gradients of the gathered tensor are summed and cut along the batch
// Both are plain copy / add kernels bound by HBM bandwidth; the part tables travel in the kernel
// arguments, so nothing is allocated and nothing is copied to the device beforehand.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/whalesplit.h"

namespace ws {

constexpr int MAXP = WS_BRIDGE_MAX_PARTS;

struct GatherTable {
    const char* src[MAXP];
    int64_t src_pitch[MAXP];     // bytes
    int64_t dst_offset[MAXP];    // bytes from `out` to the part's first element
    int32_t rows[MAXP];
    int32_t row_bytes[MAXP];
};

// Calls f(row, unit) for every unit of a rows x per_row matrix, spread over the workgroups of
// gridDim.x: wide rows are walked one row per workgroup and turn, narrow rows several at a time.
template <typename F>
__device__ __forceinline__ void for_each_unit(int rows, int per_row, F f) {
    const int nt = blockDim.x;
    if (per_row >= nt) {
        for (int r = blockIdx.x; r < rows; r += gridDim.x)
            for (int c = threadIdx.x; c < per_row; c += nt) f(r, c);
    } else if (per_row > 0) {
        const int rpb = nt / per_row;
        const int rl = (int)threadIdx.x / per_row, c = (int)threadIdx.x - rl * per_row;
        if (rl < rpb)
            for (int64_t r = (int64_t)blockIdx.x * rpb + rl; r < rows; r += (int64_t)gridDim.x * rpb) f((int)r, c);
    }
}

// Part blockIdx.y, copied in units of V bytes; the host picks the widest V that every address,
// pitch and row length of the call allows.
template <typename V>
__global__ __launch_bounds__(256) void bridge_gather_kernel(GatherTable t, char* __restrict__ out, int64_t dst_pitch) {
    const int p = blockIdx.y;
    const char* src = t.src[p];
    char* dst = out + t.dst_offset[p];
    const int64_t sp = t.src_pitch[p];
    for_each_unit(t.rows[p], t.row_bytes[p] / (int)sizeof(V), [&](int r, int c) {
        const V v = *reinterpret_cast<const V*>(src + r * sp + c * (int64_t)sizeof(V));
        *reinterpret_cast<V*>(dst + r * dst_pitch + c * (int64_t)sizeof(V)) = v;
    });
}

struct ReduceTable {
    const float* part[MAXP];
    int64_t ld_part[MAXP];       // elements
    float* out[MAXP];
    int64_t ld_out[MAXP];        // elements
    int32_t row0[MAXP];          // first row of replica r in the gathered tensor
    int32_t rows[MAXP];
};

// Replica blockIdx.y: out_r[i][d] = sum over shards s = 0 .. S-1, in that order, of
// part_s[row0_r + i][d]; one float4 per thread and turn.
__global__ __launch_bounds__(256) void bridge_reduce_partition_kernel(ReduceTable t, int S, int D4) {
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const int r = blockIdx.y;
    const int64_t row0 = t.row0[r];
    for_each_unit(t.rows[r], D4, [&](int row, int c) {
        const int64_t d = 4 * (int64_t)c;
        f32x4 s = *reinterpret_cast<const f32x4*>(t.part[0] + (row0 + row) * t.ld_part[0] + d);
        for (int k = 1; k < S; ++k) s += *reinterpret_cast<const f32x4*>(t.part[k] + (row0 + row) * t.ld_part[k] + d);
        *reinterpret_cast<f32x4*>(t.out[r] + row * t.ld_out[r] + d) = s;
    });
}

static inline bool is_aligned(uint64_t v, uint64_t a) { return (v & (a - 1)) == 0; }

// Workgroups along x for parts of at most `rows` rows of `per_row` units (see for_each_unit).
static inline unsigned grid_x(int64_t rows, int64_t per_row) {
    int64_t b = per_row >= 256 ? rows : (rows + 256 / (per_row > 0 ? per_row : 1) - 1) / (256 / (per_row > 0 ? per_row : 1));
    if (b < 1) b = 1;
    return (unsigned)(b > 2048 ? 2048 : b);      // the loops stride beyond that: 8 workgroups per CU are plenty
}

}  // namespace ws

using namespace ws;

extern "C" {

int ws_bridge_gather(int32_t dim, const void* const* parts, const int64_t* ld_parts, const int32_t* extents, int32_t n,
                     int32_t other, int32_t elem_bytes, void* out, int64_t ld_out, void* stream) {
    if (!parts || !ld_parts || !extents || !out) return WS_ERR_NULL;
    if (dim != 0 && dim != 1) return WS_ERR_RANGE;
    if (n < 1 || n > MAXP) return WS_ERR_RANGE;
    if (other <= 0 || (elem_bytes != 2 && elem_bytes != 4)) return WS_ERR_SHAPE;
    int64_t total = 0;
    for (int p = 0; p < n; ++p) {
        if (extents[p] < 0) return WS_ERR_SHAPE;
        if (extents[p] > 0 && !parts[p]) return WS_ERR_NULL;
        const int64_t cols = dim == 0 ? other : extents[p];
        if (ld_parts[p] < cols) return WS_ERR_SHAPE;
        total += extents[p];
    }
    if (total > INT32_MAX) return WS_ERR_RANGE;
    if (ld_out < (dim == 0 ? (int64_t)other : total)) return WS_ERR_SHAPE;
    if (total == 0) return WS_OK;

    GatherTable t;
    const int64_t dst_pitch = ld_out * elem_bytes;
    uint64_t bits = (uint64_t)reinterpret_cast<uintptr_t>(out) | (uint64_t)dst_pitch;    // OR of everything that must divide
    int64_t at = 0;
    int64_t max_rows = 0, max_row_bytes = 0;
    for (int p = 0; p < MAXP; ++p) {
        if (p >= n) {
            t.src[p] = nullptr; t.src_pitch[p] = 0; t.dst_offset[p] = 0; t.rows[p] = 0; t.row_bytes[p] = 0;
            continue;
        }
        const int64_t rows = dim == 0 ? extents[p] : other;
        const int64_t row_bytes = (int64_t)(dim == 0 ? other : extents[p]) * elem_bytes;
        if (row_bytes > INT32_MAX) return WS_ERR_RANGE;
        t.src[p] = static_cast<const char*>(parts[p]);
        t.src_pitch[p] = ld_parts[p] * elem_bytes;
        t.dst_offset[p] = dim == 0 ? at * dst_pitch : at * elem_bytes;
        t.rows[p] = (int32_t)rows;
        t.row_bytes[p] = (int32_t)row_bytes;
        if (extents[p] > 0) {
            bits |= (uint64_t)reinterpret_cast<uintptr_t>(parts[p]) | (uint64_t)t.src_pitch[p] |
                    (uint64_t)t.dst_offset[p] | (uint64_t)row_bytes;
            if (rows > max_rows) max_rows = rows;
            if (row_bytes > max_row_bytes) max_row_bytes = row_bytes;
        }
        at += extents[p];
    }
    if (!is_aligned(bits, (uint64_t)elem_bytes)) return WS_ERR_ALIGN;

    hipStream_t s = static_cast<hipStream_t>(stream);
    char* o = static_cast<char*>(out);
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    // x extent for the part with the most rows; narrow parts are packed by the kernel, never slower
    const unsigned gx = grid_x(max_rows, max_row_bytes >= 4096 ? 256 : max_row_bytes / 16 + 1);
    if (is_aligned(bits, 16))
        hipLaunchKernelGGL(bridge_gather_kernel<u32x4>, dim3(gx, n), dim3(256), 0, s, t, o, dst_pitch);
    else if (is_aligned(bits, 8))
        hipLaunchKernelGGL(bridge_gather_kernel<u32x2>, dim3(gx, n), dim3(256), 0, s, t, o, dst_pitch);
    else if (is_aligned(bits, 4))
        hipLaunchKernelGGL(bridge_gather_kernel<uint32_t>, dim3(gx, n), dim3(256), 0, s, t, o, dst_pitch);
    else
        hipLaunchKernelGGL(bridge_gather_kernel<uint16_t>, dim3(gx, n), dim3(256), 0, s, t, o, dst_pitch);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

int ws_bridge_reduce_partition(const float* const* partials, const int64_t* ld_partials, int32_t S, int32_t D,
                               float* const* out_parts, const int64_t* ld_out, const int32_t* rows, int32_t R,
                               void* stream) {
    if (!partials || !ld_partials || !out_parts || !ld_out || !rows) return WS_ERR_NULL;
    if (S < 1 || S > MAXP || R < 1 || R > MAXP) return WS_ERR_RANGE;
    if (D <= 0 || D % 4 != 0) return WS_ERR_SHAPE;
    ReduceTable t;
    int64_t at = 0, max_rows = 0;
    for (int r = 0; r < MAXP; ++r) {
        if (r >= R) {
            t.out[r] = nullptr; t.ld_out[r] = 0; t.row0[r] = 0; t.rows[r] = 0;
            continue;
        }
        if (rows[r] < 0) return WS_ERR_SHAPE;
        if (rows[r] > 0 && !out_parts[r]) return WS_ERR_NULL;
        if (ld_out[r] < D) return WS_ERR_SHAPE;
        if (rows[r] > 0 && (!is_aligned(reinterpret_cast<uintptr_t>(out_parts[r]), 16) || ld_out[r] % 4)) return WS_ERR_ALIGN;
        t.out[r] = out_parts[r]; t.ld_out[r] = ld_out[r]; t.row0[r] = (int32_t)at; t.rows[r] = rows[r];
        at += rows[r];
        if (rows[r] > max_rows) max_rows = rows[r];
        if (at > INT32_MAX) return WS_ERR_RANGE;
    }
    for (int k = 0; k < MAXP; ++k) {
        if (k >= S) {
            t.part[k] = nullptr; t.ld_part[k] = 0;
            continue;
        }
        if (!partials[k]) return WS_ERR_NULL;
        if (ld_partials[k] < D) return WS_ERR_SHAPE;
        if (!is_aligned(reinterpret_cast<uintptr_t>(partials[k]), 16) || ld_partials[k] % 4) return WS_ERR_ALIGN;
        t.part[k] = partials[k]; t.ld_part[k] = ld_partials[k];
    }
    if (at == 0) return WS_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(bridge_reduce_partition_kernel, dim3(grid_x(max_rows, D / 4), R), dim3(256), 0, s, t, S, D / 4);
    return hipGetLastError() == hipSuccess ? WS_OK : WS_ERR_HIP;
}

int ws_bridge_fusable(int32_t gather_dim, int32_t n_src, const int64_t* src_extents, int32_t partition_dim,
                      int32_t n_dst, const int64_t* dst_extents, int32_t* fusable) {
    if (!src_extents || !dst_extents || !fusable) return WS_ERR_NULL;
    if (n_src < 1 || n_dst < 1) return WS_ERR_RANGE;
    if (gather_dim < 0 || partition_dim < 0) return WS_ERR_RANGE;
    for (int i = 0; i < n_src; ++i)
        if (src_extents[i] < 0) return WS_ERR_SHAPE;
    for (int i = 0; i < n_dst; ++i)
        if (dst_extents[i] < 0) return WS_ERR_SHAPE;
    int ok = gather_dim == partition_dim && n_src == n_dst;
    for (int i = 0; ok && i < n_src; ++i) ok = src_extents[i] == dst_extents[i];
    *fusable = ok;
    return WS_OK;
}

}  // extern "C"
