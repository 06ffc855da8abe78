// select_topk: indices of the K largest scores, ascending (paper Sec. 3.1, "Token Selection":
// keep the top K while preserving temporal order).  Ties at the K-th value go to the lowest
// index, which is what a stable sort by (score desc, index asc) gives.
//
// N is at most a few hundred thousand (<= 512 KB of scores), so the problem is latency-bound:
// one 1024-lane workgroup does an MSB radix select on the order-preserving integer image of
// the floats (11 + 11 + 10 bits, histogram in LDS), which yields the exact K-th value and how
// many of its duplicates to keep, then one ordered pass (ballot-free packed prefix sums) writes
// the surviving indices.  No global atomics, no scratch memory, bit-exact and deterministic.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;
constexpr int kBins = 2048;

// Monotone map float -> uint32 (larger float = larger key); -0.0 is folded onto +0.0.
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t b = __float_as_uint(f);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exclusive prefix sum of one value per thread over the workgroup; `total` gets the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_sums, uint32_t &total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
    }
    __syncthreads();  // wave_sums may still be read from the previous call
    if (lane == kWave - 1) wave_sums[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    total = tot;
    return base + inc - v;
}

// After a histogram pass: find the bin (scanning from the top) that holds the k-th largest key
// and reduce k to its rank inside that bin.  All threads return the same (bin, k).
__device__ __forceinline__ void pick_bin(const uint32_t *hist, uint32_t *wave_sums, uint32_t *shared2,
                                         uint32_t &k, uint32_t &bin) {
    const int d0 = kBins - 1 - 2 * threadIdx.x, d1 = d0 - 1;  // two bins per thread, descending
    const uint32_t c0 = hist[d0], c1 = hist[d1];
    uint32_t total;
    const uint32_t above = block_exclusive_scan(c0 + c1, wave_sums, total);
    if (above < k && k <= above + c0) {
        shared2[0] = (uint32_t)d0;
        shared2[1] = k - above;
    } else if (above + c0 < k && k <= above + c0 + c1) {
        shared2[0] = (uint32_t)d1;
        shared2[1] = k - above - c0;
    }
    __syncthreads();
    bin = shared2[0];
    k = shared2[1];
    __syncthreads();
}

__global__ __launch_bounds__(kThreads) void select_topk_kernel(const float *__restrict__ scores, int N, int K,
                                                               int32_t *__restrict__ idx) {
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wave_sums[kWaves];
    __shared__ uint32_t shared2[2];
    const int tid = threadIdx.x;

    // ---- radix select: exact key of the K-th largest score --------------------------------
    uint32_t k = (uint32_t)K, prefix = 0, bin;
    // pass 0: top 11 bits
    for (int b = tid; b < kBins; b += kThreads) hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) atomicAdd(&hist[order_key(scores[i]) >> 21], 1u);
    __syncthreads();
    pick_bin(hist, wave_sums, shared2, k, bin);
    prefix = bin << 21;
    // pass 1: middle 11 bits of the keys that share the top 11
    for (int b = tid; b < kBins; b += kThreads) hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
        const uint32_t key = order_key(scores[i]);
        if ((key >> 21) == (prefix >> 21)) atomicAdd(&hist[(key >> 10) & 0x7FFu], 1u);
    }
    __syncthreads();
    pick_bin(hist, wave_sums, shared2, k, bin);
    prefix |= bin << 10;
    // pass 2: low 10 bits
    for (int b = tid; b < kBins; b += kThreads) hist[b] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
        const uint32_t key = order_key(scores[i]);
        if ((key >> 10) == (prefix >> 10)) atomicAdd(&hist[key & 0x3FFu], 1u);
    }
    __syncthreads();
    pick_bin(hist, wave_sums, shared2, k, bin);
    const uint32_t thresh = prefix | bin;  // key of the K-th largest score
    const uint32_t keep_eq = k;            // how many keys == thresh survive (the first ones)

    // ---- ordered write-out: 4 consecutive scores per thread per tile ------------------------
    uint32_t out_base = 0, eq_base = 0;    // survivors / duplicates of thresh seen in earlier tiles
    for (int t0 = 0; t0 < N; t0 += kThreads * 4) {
        const int i0 = t0 + tid * 4;
        uint32_t key[4];
        uint32_t cnt = 0;  // low 16 bits: keys > thresh, high 16 bits: keys == thresh
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            key[u] = (i0 + u < N) ? order_key(scores[i0 + u]) : 0u;
            const bool in = i0 + u < N;
            cnt += (in && key[u] > thresh) ? 1u : 0u;
            cnt += (in && key[u] == thresh) ? 0x10000u : 0u;
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan(cnt, wave_sums, total);
        uint32_t gt_before = ex & 0xFFFFu, eq_before = eq_base + (ex >> 16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u < N) {
                const bool gt = key[u] > thresh, eq = key[u] == thresh;
                if (gt || (eq && eq_before < keep_eq)) {
                    const uint32_t eq_kept = min(eq_before, keep_eq) - min(eq_base, keep_eq);
                    idx[out_base + gt_before + eq_kept] = i0 + u;
                }
                gt_before += gt ? 1u : 0u;
                eq_before += eq ? 1u : 0u;
            }
        }
        const uint32_t eq_tile = total >> 16;
        out_base += (total & 0xFFFFu) + (min(eq_base + eq_tile, keep_eq) - min(eq_base, keep_eq));
        eq_base += eq_tile;
    }
}

}  // namespace

int select_topk_launch(const float *scores, int N, int K, int32_t *idx, hipStream_t s) {
    select_topk_kernel<<<1, kThreads, 0, s>>>(scores, N, K, idx);
    return launch_status();
}

}  // namespace strd
