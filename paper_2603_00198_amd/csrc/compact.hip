// compact: order-preserving row gather of per-token tensors (paper Sec. 3.1, token selection:
// retained vision tokens continue, the text tail is kept whole).
// Pure HBM-bound copy: every lane moves 16-byte vectors (non-temporal loads, cached stores), the
// loads of a thread are issued before its stores, consecutive lanes touch consecutive vectors of a row.  Up to
// STRD_COMPACT_MAX tensors that share one index list are gathered by a single launch
// (blockIdx.y selects the tensor), which matters because a reduced layer compacts 4-5 tensors
// of a few tens of MB each and a launch costs about as much as moving 20 MB.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
constexpr int kVecPerThread = 2;  // about this many vectors per thread: whole rows per workgroup, or a piece of a row
                                  // longer than that (many small workgroups measured 5-7 % faster than 8 or 16
                                  // vectors per thread, and 16 KB rows 4 % faster in two pieces than whole; one
                                  // vector per thread is 15 % slower)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct Item {
    const void *src;
    void *dst;
    int vec_per_row;     // row length in vectors
    int rows_per_block;  // whole rows handled by one workgroup (1 when blocks_per_row > 1)
    int blocks_per_row;  // workgroups that share one row: a row longer than a workgroup's share is cut into pieces
    int vec16;           // 1: 16-byte vectors, 0: 4-byte vectors
    int identity;        // 1: write the source row number itself (position map without pos_in)
};
struct Batch {
    Item item[STRD_COMPACT_MAX + 1];
    int first_block[STRD_COMPACT_MAX + 2];  // workgroups [first_block[i], first_block[i + 1]) belong to item i
    int n_items;
    int grid;  // workgroups of all items together
    // 1: the launch writes more than the last-level cache (256 MB) holds, so nothing of it would still be
    // there when the mixer reads it: non-temporal stores (-6 % at 131072 tokens; +7 % at 32768, where the
    // 173 MB written do fit, hence the switch)
    int stream_out;
};
// The item a workgroup belongs to and its number among that item's workgroups (uniform).
// (entries past the last item hold INT_MAX: all bounds are fetched at once and compared without a branch)
__device__ __forceinline__ int item_of(const Batch &b, int block, int &local) {
    int i = 0, first = 0;
#pragma unroll
    for (int j = 1; j <= STRD_COMPACT_MAX; ++j) {
        const bool past = block >= b.first_block[j];
        i += past ? 1 : 0;
        first = past ? b.first_block[j] : first;
    }
    local = block - first;
    return i;
}

// Rows of one sequence: source rows count from src_row0, output rows from dst_row0 (both 0 for a
// single sequence).
template <typename Vec>
__device__ __forceinline__ void copy_rows(const Item &it, const int32_t *__restrict__ idx, int N, int K, int rows_out,
                                          int block, bool stream_out, size_t src_row0 = 0, size_t dst_row0 = 0) {
    const int vpr = it.vec_per_row;
    const Vec *__restrict__ src = reinterpret_cast<const Vec *>(it.src) + src_row0 * vpr;
    Vec *__restrict__ dst = reinterpret_cast<Vec *>(it.dst) + dst_row0 * vpr;
    // whole rows, or (long rows) one piece of kThreads * kVecPerThread vectors of one row
    const int bpr = it.blocks_per_row;
    const int row0 = bpr > 1 ? block / bpr : block * it.rows_per_block;
    const int col0 = bpr > 1 ? (block - row0 * bpr) * (kThreads * kVecPerThread) : 0;
    if (row0 >= rows_out) return;
    const int nrows = min(it.rows_per_block, rows_out - row0);
    const int total = bpr > 1 ? min(kThreads * kVecPerThread, vpr - col0) : nrows * vpr;
    for (int e0 = threadIdx.x; e0 < total; e0 += kThreads * kUnroll) {
        Vec v[kUnroll];
        size_t off[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int e = e0 + u * kThreads;
            if (e < total) {
                const int rl = bpr > 1 ? 0 : e / vpr;
                const int c = bpr > 1 ? col0 + e : e - rl * vpr;
                const int r = row0 + rl;
                const int sr = (r < K) ? idx[r] : (N + (r - K));
                v[u] = __builtin_nontemporal_load(src + (size_t)sr * vpr + c);  // streamed once: keep it out of L2
                off[u] = (size_t)r * vpr + c;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            if (e0 + u * kThreads < total) {
                if (stream_out)
                    __builtin_nontemporal_store(v[u], dst + off[u]);  // more than the last-level cache holds
                else
                    dst[off[u]] = v[u];  // cached: the mixer reads it next
            }
    }
}

__global__ __launch_bounds__(kThreads) void compact_kernel(Batch b, const int32_t *__restrict__ idx, int N, int K,
                                                           int rows_out) {
    // one grid dimension for all tensors: every tensor gets exactly the workgroups its rows need
    int block;
    const Item &it = b.item[item_of(b, blockIdx.x, block)];
    if (it.identity) {
        const int r = block * kThreads + threadIdx.x;
        if (r < rows_out) reinterpret_cast<int32_t *>(it.dst)[r] = (r < K) ? idx[r] : (N + (r - K));
    } else if (it.vec16) {
        copy_rows<u32x4>(it, idx, N, K, rows_out, block, b.stream_out != 0);
    } else {
        copy_rows<uint32_t>(it, idx, N, K, rows_out, block, b.stream_out != 0);
    }
}

// Packed batch: blockIdx.z selects the sequence.  Positions are local to the sequence (row number
// among its own N + M input rows), or pos_in of that row.
__global__ __launch_bounds__(kThreads) void compact_varlen_kernel(Batch b, const int32_t *__restrict__ idx, SeqTab tab) {
    const Item &it = b.item[blockIdx.y];
    const int q = blockIdx.z;
    const int N = tab.N[q], K = tab.K[q], rows_out = K + tab.M[q];
    const int32_t *ix = idx + tab.koff[q];
    if (it.identity) {
        const int r = blockIdx.x * kThreads + threadIdx.x;
        if (r < rows_out) reinterpret_cast<int32_t *>(it.dst)[tab.ooff[q] + r] = (r < K) ? ix[r] : (N + (r - K));
    } else if (it.vec16) {
        copy_rows<u32x4>(it, ix, N, K, rows_out, blockIdx.x, b.stream_out != 0, tab.row0[q], tab.ooff[q]);
    } else {
        copy_rows<uint32_t>(it, ix, N, K, rows_out, blockIdx.x, b.stream_out != 0, tab.row0[q], tab.ooff[q]);
    }
}

}  // namespace

// Fills the launch table from the caller's items; returns the grid width for `rows_out` output rows.
static int compact_plan(const strd_compact_item *items, int n_items, const int32_t *pos_in, int32_t *pos_out,
                        int rows_out, int nseq_hint, Batch &b, int &n, int &grid_x) {
    n = 0;
    grid_x = 1;
    for (int i = 0; i < n_items; ++i) {
        const strd_compact_item &ci = items[i];
        Item it;
        it.src = ci.src;
        it.dst = ci.dst;
        it.identity = 0;
        it.vec16 = (ci.row_bytes % 16 == 0) && ((uintptr_t)ci.src % 16 == 0) && ((uintptr_t)ci.dst % 16 == 0);
        const int64_t vpr = it.vec16 ? ci.row_bytes / 16 : ci.row_bytes / 4;
        if (vpr > (1 << 26)) return STRD_EUNSUPPORTED;
        it.vec_per_row = (int)vpr;
        // whole rows per workgroup, or several workgroups per row: about kVecPerThread vectors per thread either way
        it.rows_per_block = (kThreads * kVecPerThread) / it.vec_per_row;
        if (it.rows_per_block < 1) it.rows_per_block = 1;
        it.blocks_per_row = ceil_div(it.vec_per_row, kThreads * kVecPerThread);
        const long long blocks = it.blocks_per_row > 1 ? (long long)rows_out * it.blocks_per_row
                                                       : (long long)ceil_div(rows_out, it.rows_per_block);
        if (blocks > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
        grid_x = max(grid_x, (int)blocks);
        b.first_block[n + 1] = (int)blocks;
        b.item[n++] = it;
    }
    if (pos_out) {
        Item it;
        it.src = pos_in;
        it.dst = pos_out;
        it.identity = pos_in ? 0 : 1;
        it.vec16 = 0;
        it.vec_per_row = 1;
        it.blocks_per_row = 1;
        it.rows_per_block = kThreads * 8;
        grid_x = max(grid_x, ceil_div(rows_out, pos_in ? it.rows_per_block : kThreads));
        b.first_block[n + 1] = ceil_div(rows_out, pos_in ? it.rows_per_block : kThreads);
        b.item[n++] = it;
    }
    // per-item counts -> running totals (used by the single-sequence launch, which has one grid dimension)
    b.first_block[0] = 0;
    long long total = 0;
    for (int i = 0; i < n; ++i) {
        total += b.first_block[i + 1];
        if (total > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
        b.first_block[i + 1] = (int)total;
    }
    const int grid = b.first_block[n];
    long long bytes = 0;
    for (int i = 0; i < n_items; ++i) bytes += (long long)rows_out * items[i].row_bytes;
    b.stream_out = bytes * (long long)(nseq_hint > 0 ? nseq_hint : 1) > 256LL * 1024 * 1024 ? 1 : 0;
    for (int i = n; i <= STRD_COMPACT_MAX + 1; ++i) b.first_block[i] = 0x7FFFFFFF;
    b.n_items = n;
    b.grid = grid;
    return STRD_OK;
}

int compact_varlen_launch(const strd_compact_item *items, int n_items, const int32_t *idx, const SeqTab &tab, int nseq,
                          int max_rows_out, const int32_t *pos_in, int32_t *pos_out, hipStream_t s) {
    if (max_rows_out == 0 || nseq == 0) return STRD_OK;
    Batch b;
    int n, grid_x;
    const int rc = compact_plan(items, n_items, pos_in, pos_out, max_rows_out, nseq, b, n, grid_x);
    if (rc != STRD_OK) return rc;
    if (n == 0) return STRD_OK;
    compact_varlen_kernel<<<dim3(grid_x, n, nseq), kThreads, 0, s>>>(b, idx, tab);
    return launch_status();
}

int compact_launch(const strd_compact_item *items, int n_items, const int32_t *idx, int N, int M, int K,
                   const int32_t *pos_in, int32_t *pos_out, hipStream_t s) {
    const int rows_out = K + M;
    if (rows_out == 0) return STRD_OK;
    Batch b;
    int n, grid_x;
    const int rc = compact_plan(items, n_items, pos_in, pos_out, rows_out, 1, b, n, grid_x);
    if (rc != STRD_OK) return rc;
    if (n == 0) return STRD_OK;
    compact_kernel<<<b.grid, kThreads, 0, s>>>(b, idx, N, K, rows_out);
    return launch_status();
}

}  // namespace strd
