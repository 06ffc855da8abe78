// compact: order-preserving row gather of one per-token tensor (paper Sec. 3.1, token
// selection: retained vision tokens continue, the text tail is kept whole).
// Pure HBM-bound copy: every lane moves 16-byte vectors, the loads of a thread are issued
// before its stores, consecutive lanes touch consecutive vectors of a row.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

// One workgroup copies `rows_per_block` consecutive destination rows.  Vec is uint4 (rows a
// multiple of 16 bytes) or uint32_t.
template <typename Vec>
__global__ __launch_bounds__(kThreads) void compact_rows_kernel(
    const Vec *__restrict__ src, const int32_t *__restrict__ idx, Vec *__restrict__ dst, int N, int K,
    int rows_out, int vec_per_row, int rows_per_block) {
    const int row0 = blockIdx.x * rows_per_block;
    const int nrows = min(rows_per_block, rows_out - row0);
    const int total = nrows * vec_per_row;
    for (int e0 = threadIdx.x; e0 < total; e0 += kThreads * kUnroll) {
        Vec v[kUnroll];
        size_t off[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int e = e0 + u * kThreads;
            if (e < total) {
                const int rl = e / vec_per_row;
                const int c = e - rl * vec_per_row;
                const int r = row0 + rl;
                const int sr = (r < K) ? idx[r] : (N + (r - K));
                v[u] = src[(size_t)sr * vec_per_row + c];
                off[u] = (size_t)r * vec_per_row + c;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            if (e0 + u * kThreads < total) dst[off[u]] = v[u];
    }
}

__global__ __launch_bounds__(kThreads) void compact_pos_kernel(const int32_t *__restrict__ idx,
                                                               const int32_t *__restrict__ pos_in,
                                                               int32_t *__restrict__ pos_out, int N,
                                                               int K, int rows_out) {
    const int r = blockIdx.x * kThreads + threadIdx.x;
    if (r >= rows_out) return;
    const int sr = (r < K) ? idx[r] : (N + (r - K));
    pos_out[r] = pos_in ? pos_in[sr] : sr;
}

}  // namespace

int compact_launch(const void *src, const int32_t *idx, void *dst, int N, int M, int K,
                   int64_t row_bytes, const int32_t *pos_in, int32_t *pos_out, hipStream_t s) {
    const int rows_out = K + M;
    if (rows_out == 0) return STRD_OK;
    if (src && dst) {
        const bool v16 = (row_bytes % 16 == 0) && ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0);
        const int64_t vpr64 = v16 ? row_bytes / 16 : row_bytes / 4;
        if (vpr64 > (1 << 26)) return STRD_EUNSUPPORTED;
        const int vpr = (int)vpr64;
        // about 8 vectors per thread per workgroup, whole rows only
        int rpb = (kThreads * 8) / vpr;
        if (rpb < 1) rpb = 1;
        const int grid = ceil_div(rows_out, rpb);
        if (v16)
            compact_rows_kernel<uint4><<<grid, kThreads, 0, s>>>((const uint4 *)src, idx, (uint4 *)dst, N, K,
                                                                 rows_out, vpr, rpb);
        else
            compact_rows_kernel<uint32_t><<<grid, kThreads, 0, s>>>((const uint32_t *)src, idx,
                                                                    (uint32_t *)dst, N, K, rows_out, vpr, rpb);
        if (launch_status() != STRD_OK) return STRD_EHIP;
    }
    if (pos_out) {
        compact_pos_kernel<<<ceil_div(rows_out, kThreads), kThreads, 0, s>>>(idx, pos_in, pos_out, N, K, rows_out);
        if (launch_status() != STRD_OK) return STRD_EHIP;
    }
    return STRD_OK;
}

}  // namespace strd
