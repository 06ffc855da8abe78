// select_topk: indices of the K largest scores, ascending (paper Sec. 3.1, "Token Selection":
// keep the top K while preserving temporal order).  Ties at the K-th value go to the lowest
// index, which is what a stable sort by (score desc, index asc) gives.
//
// N is at most a few hundred thousand (<= 512 KB of scores), so the problem is latency-bound.
// Up to 32768 scores (and beyond 2^20, streaming) one 1024-lane workgroup does everything in one
// launch; between the two a chain of six short launches with one workgroup per 4096 scores is
// three to four times faster than streaming (see "Wide form" below).
// The one-launch form: an MSB radix select on the order-preserving integer image of
// the floats, which yields the exact K-th value and how many of its duplicates to keep, then one
// ordered pass (packed prefix sums) writes the surviving indices.  The digits (11 bits each,
// histogram in LDS) are taken from key - min(key): the scores of a layer lie close together, so
// the leading bits of the raw keys carry no information, while the significant bits of the
// offsets usually fit two passes and spread over the bins.  Each lane owns 4 consecutive scores
// of every 4096-score tile; up to 32768 scores the keys are read from memory once and stay in
// registers for all passes, beyond that they are re-read in batches of 8 tiles with all loads of
// a batch in flight together.  Same-address LDS atomics serialise, so in the first pass every bin
// has 16 copies, one per lane modulo 16, in adjacent LDS words (different banks), summed when a
// bin is picked; later passes only count the keys of one bin of the pass before and use 2 copies
// when those are few; once a bin holds no more than one wave's worth of keys the remaining digits
// are skipped and one wave ranks those keys directly.  The ordered pass scans 8 tiles per barrier.  No global atomics, no
// scratch memory, bit-exact and deterministic.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;
constexpr int kBins = 2048;
constexpr int kTile = kThreads * 4;  // scores per tile
constexpr int kBatch = 8;            // tiles loaded together when streaming / scanned per barrier
constexpr int kCopies = 16;          // copies of every histogram bin
constexpr int kFewCopies = 2;        // copies in passes 1 and 2 when at most kFewKeys keys are still in play
constexpr int kFewKeys = 4096;
constexpr int kRankKeys = 64;        // at most this many keys still in play: one wave ranks them directly

// Monotone map float -> uint32 (larger float = larger key); -0.0 is folded onto +0.0.
// Every score maps above 0, the key given to the slots past the end of the array: the one bit
// pattern whose image would be 0 (a negative NaN, all bits set) shares key 1 with its neighbour,
// so that exactly K indices are written whatever the input holds.  NaNs are ordered by their
// bits: positive ones above +inf, negative ones below -inf.
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t b = __float_as_uint(f);
    if (b == 0x80000000u) b = 0u;
    return max((b & 0x80000000u) ? ~b : (b | 0x80000000u), 1u);
}

// Keys of the 4 scores this lane owns in tile `t` (0 past the end).
__device__ __forceinline__ void load_tile(const float *__restrict__ scores, int N, int t, uint32_t (&key)[4]) {
    const int i0 = t * kTile + threadIdx.x * 4;
    if (i0 + 3 < N) {
        const float4 v = *reinterpret_cast<const float4 *>(scores + i0);
        key[0] = order_key(v.x); key[1] = order_key(v.y); key[2] = order_key(v.z); key[3] = order_key(v.w);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) key[u] = (i0 + u < N) ? order_key(scores[i0 + u]) : 0u;
    }
}

// hist[bin] += 1 in this lane's copy of the bin (COPIES copies per bin, adjacent words).
template <int COPIES>
__device__ __forceinline__ void hist_add(uint32_t *hist, uint32_t bin, bool valid) {
    if (valid) atomicAdd(&hist[bin * COPIES + (threadIdx.x & (COPIES - 1))], 1u);
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves (no LDS round trips):
// Kogge-Stone inside each row of 16 lanes, then the row totals are broadcast forward.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
#define STRD_DPP_ADD(ctrl, row_mask) \
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, row_mask, 0xF, true)
    STRD_DPP_ADD(0x111, 0xF);  // row_shr:1
    STRD_DPP_ADD(0x112, 0xF);  // row_shr:2
    STRD_DPP_ADD(0x114, 0xF);  // row_shr:4
    STRD_DPP_ADD(0x118, 0xF);  // row_shr:8
    STRD_DPP_ADD(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
    STRD_DPP_ADD(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef STRD_DPP_ADD
    return v;
}

// Cross-wave step of up to kBatch workgroup scans that share one pair of barriers.  Before the
// call every wave has stored the inclusive total of scan b in sums[b][wave].  The first 16*kBatch
// threads turn each row of 16 wave totals into exclusive offsets with a DPP row scan (a row of
// 16 lanes is exactly one scan) and append the grand total as element [b][kWaves].
struct ScanScratch {
    uint32_t sums[kBatch][kWaves];
    uint32_t base[kBatch][kWaves + 1];
};
__device__ __forceinline__ void finish_scans(ScanScratch &sc) {
    __syncthreads();
    if (threadIdx.x < kBatch * kWaves) {
        const int b = threadIdx.x / kWaves, w = threadIdx.x % kWaves;
        const uint32_t v = sc.sums[b][w];
        uint32_t inc = v;
#define STRD_DPP_ADD(ctrl) inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, ctrl, 0xF, 0xF, true)
        STRD_DPP_ADD(0x111);
        STRD_DPP_ADD(0x112);
        STRD_DPP_ADD(0x114);
        STRD_DPP_ADD(0x118);
#undef STRD_DPP_ADD
        sc.base[b][w] = inc - v;
        if (w == kWaves - 1) sc.base[b][kWaves] = inc;
    }
    __syncthreads();
}

// After a histogram pass: find the bin (scanning from the top) that holds the k-th largest key
// and reduce k to its rank inside that bin.  All threads return the same (bin, k).  Thread t owns
// bins 2047 - t and 1023 - t, so neighbouring threads read neighbouring 64-byte groups of copies.
template <int COPIES>
__device__ __forceinline__ void pick_bin(const uint32_t *hist, ScanScratch &sc, uint32_t *found, uint32_t &k,
                                         uint32_t &bin) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int d_hi = kBins - 1 - threadIdx.x, d_lo = d_hi - kThreads;
    uint32_t c_hi = 0, c_lo = 0;
    if (COPIES >= 4) {
#pragma unroll
        for (int c = 0; c < COPIES; c += 4) {
            const uint4 a = *reinterpret_cast<const uint4 *>(&hist[d_hi * COPIES + c]);
            const uint4 b = *reinterpret_cast<const uint4 *>(&hist[d_lo * COPIES + c]);
            c_hi += a.x + a.y + a.z + a.w;
            c_lo += b.x + b.y + b.z + b.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < COPIES; ++c) {
            c_hi += hist[d_hi * COPIES + c];
            c_lo += hist[d_lo * COPIES + c];
        }
    }
    const uint32_t i_hi = wave_inclusive_scan(c_hi), i_lo = wave_inclusive_scan(c_lo);
    if (lane == kWave - 1) {
        sc.sums[0][wave] = i_hi;
        sc.sums[1][wave] = i_lo;
    }
    finish_scans(sc);
    // keys in higher bins than this thread's: all upper-half bins come before any lower-half bin
    const uint32_t above_hi = sc.base[0][wave] + i_hi - c_hi;
    const uint32_t above_lo = sc.base[0][kWaves] + sc.base[1][wave] + i_lo - c_lo;
    if (above_hi < k && k <= above_hi + c_hi) {
        found[0] = (uint32_t)d_hi;
        found[1] = k - above_hi;
        found[2] = c_hi;
    } else if (above_lo < k && k <= above_lo + c_lo) {
        found[0] = (uint32_t)d_lo;
        found[1] = k - above_lo;
        found[2] = c_lo;
    }
    __syncthreads();
    bin = found[0];
    k = found[1];
}

// TILES > 0: N <= TILES * kTile and every key stays in registers.  TILES == 0: streaming.
// SEQ = SeqTab: one workgroup per sequence of a packed batch (scores of sequence b start at
// scores + b * ld, its indices at idx + koff[b]; N and K are the table's).
template <int TILES, class SEQ = OneSeq>
__global__ __launch_bounds__(kThreads) void select_topk_kernel(const float *__restrict__ scores, int N, int K,
                                                               int32_t *__restrict__ idx, SEQ seq, int ld) {
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.x;
        N = seq.N[b];
        K = seq.K[b];
        scores += (size_t)b * ld;
        idx += seq.koff[b];
    }
    extern __shared__ __attribute__((aligned(16))) uint32_t hist[];  // [kBins][kCopies]
    __shared__ ScanScratch scan;
    __shared__ uint32_t found[3][3];         // (bin, rank inside the bin, keys in the bin) of each pass
    __shared__ uint32_t cand[kRankKeys];     // direct ranking: the keys (less kmin) still in play
    __shared__ uint32_t ncand, ranked_key[2];
    const int tid = threadIdx.x;
    if (tid == 0) ncand = 0u;                // published by the first barrier below
    const int ntiles = (N + kTile - 1) / kTile;
    auto zero_hist = [&](int copies) {
        for (int b = tid * 4; b < kBins * copies; b += kThreads * 4)
            *reinterpret_cast<uint4 *>(&hist[b]) = make_uint4(0, 0, 0, 0);
    };
    zero_hist(kCopies);

    constexpr int kHeld = TILES > 0 ? TILES : 1;
    uint32_t held[kHeld][4];
    if (TILES > 0) {
#pragma unroll
        for (int t = 0; t < kHeld; ++t) load_tile(scores, N, t, held[t]);
    }
    // Visit every key this lane owns; f is inlined into both variants.
    auto for_each_key = [&](auto &&f) {
        if (TILES > 0) {
#pragma unroll
            for (int t = 0; t < kHeld; ++t)
#pragma unroll
                for (int u = 0; u < 4; ++u) f(held[t][u]);
        } else {
            for (int t0 = 0; t0 < ntiles; t0 += kBatch) {
                uint32_t key[kBatch][4];
#pragma unroll
                for (int b = 0; b < kBatch; ++b) load_tile(scores, N, t0 + b, key[b]);  // past-the-end tiles give 0
#pragma unroll
                for (int b = 0; b < kBatch; ++b)
#pragma unroll
                    for (int u = 0; u < 4; ++u) f(key[b][u]);
            }
        }
    };

    // ---- radix select: exact key of the K-th largest score --------------------------------
    // Importance scores are close together (all scores of a layer within a factor of two is
    // normal), so the leading bits of the keys say nothing: the digits are taken from
    // rel = key - (smallest key) instead, whose nbits significant bits are cut into 11-bit digits
    // from the top.  Scores within a factor of two need two passes instead of three, and the keys
    // spread over the bins instead of crowding a few.
    // (When the keys do not fit the registers, finding the smallest key would cost one more pass
    // over memory, as much as the digit it may save: the raw keys are used then.)
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    if (TILES > 0) {
        for_each_key([&](uint32_t key) {
            if (key) {  // 0 marks the slots past the end of the array
                kmin = min(kmin, key);
                kmax = max(kmax, key);
            }
        });
    } else {
        kmin = 0u;
        kmax = 0xFFFFFFFFu;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, kWave));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
    }
    if ((tid & (kWave - 1)) == 0) {
        scan.sums[0][tid / kWave] = kmin;
        scan.sums[1][tid / kWave] = kmax;
    }
    __syncthreads();  // also publishes the cleared histogram
#pragma unroll
    for (int wv = 0; wv < kWaves; ++wv) {
        kmin = min(kmin, scan.sums[0][wv]);
        kmax = max(kmax, scan.sums[1][wv]);
    }
    const int nbits = 32 - __clz(kmax - kmin);     // 0 when all scores are equal
    const int npass = (nbits + 10) / 11;           // uniform
    // Pass 0 sees every key: 16 copies per bin, whatever the distribution.  A later pass only counts
    // the keys of one bin of the pass before; when those are few, their digits rarely collide and a
    // histogram with 2 copies per bin is 8 times cheaper to clear and to scan.
    uint32_t k = (uint32_t)K, prefix = 0;          // prefix: the digits of rel fixed so far, in place
    int shift_prev = 32;
    bool few = false, ranked = false;
    for (int pass = 0; pass < npass; ++pass) {
        if (pass > 0 && found[pass - 1][2] <= (uint32_t)kRankKeys) {  // uniform
            // The bin of the pass before holds a wave's worth of keys at most: collect them and let every
            // lane of wave 0 count the keys above and equal to its own -- two barriers instead of one or
            // two more histogram passes of five each.
            const uint32_t pfx = prefix >> shift_prev;
            for_each_key([&](uint32_t key) {
                const uint32_t rel = key - kmin;
                if (key != 0 && (rel >> shift_prev) == pfx) cand[atomicAdd(&ncand, 1u)] = rel;
            });
            __syncthreads();
            if (tid < kWave) {
                const uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane((int)ncand);
                const uint32_t mine = (uint32_t)tid < c ? cand[tid] : 0u;
                uint32_t above = 0, equal = 0;
                for (uint32_t j = 0; j < c; ++j) {
                    const uint32_t other = (uint32_t)__builtin_amdgcn_readlane((int)mine, (int)j);
                    above += other > mine ? 1u : 0u;
                    equal += other == mine ? 1u : 0u;
                }
                if ((uint32_t)tid < c && above < k && k <= above + equal) {  // lanes with equal keys agree
                    ranked_key[0] = mine;
                    ranked_key[1] = k - above;
                }
            }
            __syncthreads();
            ranked = true;
            break;
        }
        const int shift = max(nbits - 11 * (pass + 1), 0);
        const uint32_t dmask = (1u << min(11, nbits - 11 * pass)) - 1u;
        uint32_t bin;
        if (pass > 0) {  // every lane has read its bins before the barrier inside pick_bin
            zero_hist(few ? kFewCopies : kCopies);
            __syncthreads();
        }
        const uint32_t pfx = shift_prev < 32 ? prefix >> shift_prev : 0u;
        if (few) {
            for_each_key([&](uint32_t key) {
                const uint32_t rel = key - kmin;
                hist_add<kFewCopies>(hist, (rel >> shift) & dmask, key != 0 && (shift_prev >= 32 || (rel >> shift_prev) == pfx));
            });
            __syncthreads();
            pick_bin<kFewCopies>(hist, scan, found[pass], k, bin);
        } else {
            for_each_key([&](uint32_t key) {
                const uint32_t rel = key - kmin;
                hist_add<kCopies>(hist, (rel >> shift) & dmask, key != 0 && (shift_prev >= 32 || (rel >> shift_prev) == pfx));
            });
            __syncthreads();
            pick_bin<kCopies>(hist, scan, found[pass], k, bin);
        }
        prefix |= bin << shift;
        few = found[pass][2] <= kFewKeys;  // uniform
        shift_prev = shift;
    }
    // key of the K-th largest score (a real score: > 0) and how many keys equal to it survive (the first ones)
    const uint32_t thresh = kmin + (ranked ? ranked_key[0] : prefix);
    const uint32_t keep_eq = ranked ? ranked_key[1] : k;

    // ---- ordered write-out: kBatch tiles per barrier ----------------------------------------
    uint32_t out_base = 0, eq_base = 0;  // survivors / duplicates of thresh seen in earlier tiles
    auto emit_batch = [&](int t0, const uint32_t (&key)[kBatch][4], int ntile) {
        const int lane = tid & (kWave - 1), wave = tid / kWave;
        uint32_t cnt[kBatch], inc[kBatch];  // low 16 bits: keys > thresh, high 16 bits: keys == thresh
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            cnt[b] = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                cnt[b] += (key[b][u] > thresh ? 1u : 0u) + (key[b][u] == thresh ? 0x10000u : 0u);
            inc[b] = wave_inclusive_scan(cnt[b]);
            if (lane == kWave - 1) scan.sums[b][wave] = inc[b];
        }
        finish_scans(scan);
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            if (b < ntile) {  // uniform
                const uint32_t total = scan.base[b][kWaves];
                const uint32_t ex = scan.base[b][wave] + inc[b] - cnt[b];
                const int i0 = (t0 + b) * kTile + tid * 4;
                uint32_t gt_before = ex & 0xFFFFu, eq_before = eq_base + (ex >> 16);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool gt = key[b][u] > thresh, eq = key[b][u] == thresh;
                    if (gt || (eq && eq_before < keep_eq)) {
                        const uint32_t eq_kept = min(eq_before, keep_eq) - min(eq_base, keep_eq);
                        idx[out_base + gt_before + eq_kept] = i0 + u;
                    }
                    gt_before += gt ? 1u : 0u;
                    eq_before += eq ? 1u : 0u;
                }
                const uint32_t eq_tile = total >> 16;
                out_base += (total & 0xFFFFu) + (min(eq_base + eq_tile, keep_eq) - min(eq_base, keep_eq));
                eq_base += eq_tile;
            }
        }
    };
    if (TILES > 0) {
        uint32_t key[kBatch][4];
#pragma unroll
        for (int t0 = 0; t0 < kHeld; t0 += kBatch) {
#pragma unroll
            for (int b = 0; b < kBatch; ++b)
#pragma unroll
                for (int u = 0; u < 4; ++u) key[b][u] = (t0 + b < kHeld) ? held[t0 + b < kHeld ? t0 + b : 0][u] : 0u;
            emit_batch(t0, key, min(kBatch, ntiles - t0));
        }
    } else {
        for (int t0 = 0; t0 < ntiles; t0 += kBatch) {
            uint32_t key[kBatch][4];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) load_tile(scores, N, t0 + b, key[b]);
            emit_batch(t0, key, min(kBatch, ntiles - t0));
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Wide form, 32768 < N <= kWideMax * 4096: one workgroup per 4096-score tile and a chain of short
// launches instead of one workgroup that streams the scores four times.  The same MSB radix
// select on the raw keys (three digits of 11, 11 and 10 bits), with one histogram per digit in
// global memory that the workgroups add their local counts to; the launch that counts digit p
// first picks the bin of digit p - 1 (every workgroup for itself, from the finished histogram;
// workgroup 0 leaves the result in memory for the launches after it).  The last two launches count
// the survivors of every tile and write them out in order.  Integer atomics only: the result is
// bit-exact and deterministic.
constexpr int kWideMax = 256;   // tiles (workgroups) at most
constexpr int kWideCopies = 4;  // copies of a bin in the local histogram of one tile

struct WideWs {
    uint32_t ghist[3][kBins];       // global histograms of the three digits
    uint32_t state[3][4];           // after picking digit p: (prefix so far, rank inside the bin)
    uint32_t counts[kWideMax][2];   // per tile: keys above the threshold, keys equal to it
};

__device__ __forceinline__ int wide_shift(int pass) { return pass == 0 ? 21 : pass == 1 ? 10 : 0; }
__device__ __forceinline__ uint32_t wide_mask(int pass) { return pass == 2 ? 0x3FFu : 0x7FFu; }

__global__ __launch_bounds__(kThreads) void topk_wide_zero_kernel(WideWs *ws) {
    uint32_t *h = &ws->ghist[0][0];
    for (int i = threadIdx.x; i < 3 * kBins; i += kThreads) h[i] = 0u;
}

// Picks the bin of digit PASS - 1 from its finished global histogram; returns the prefix and rank
// after it (the same in every thread of every workgroup).
template <int PASS>
__device__ __forceinline__ void wide_pick(WideWs *ws, int K, uint32_t *pickbuf, ScanScratch &scan, uint32_t *found,
                                          uint32_t &prefix, uint32_t &k) {
    prefix = 0;
    k = (uint32_t)K;
    if (PASS > 1) {
        prefix = ws->state[PASS - 2][0];
        k = ws->state[PASS - 2][1];
    }
    for (int b = threadIdx.x; b < kBins; b += kThreads) pickbuf[b] = ws->ghist[PASS - 1][b];
    __syncthreads();
    uint32_t bin;
    pick_bin<1>(pickbuf, scan, found, k, bin);
    prefix |= bin << wide_shift(PASS - 1);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ws->state[PASS - 1][0] = prefix;
        ws->state[PASS - 1][1] = k;
    }
}

// Launch PASS = 0, 1, 2: local histogram of digit PASS over the tile's keys that carry the digits
// picked so far, added to the global histogram.
template <int PASS>
__global__ __launch_bounds__(kThreads) void topk_wide_hist_kernel(const float *__restrict__ scores, int N, int K,
                                                                    WideWs *ws) {
    __shared__ __attribute__((aligned(16))) uint32_t hist[kBins * kWideCopies];
    __shared__ uint32_t pickbuf[kBins];
    __shared__ ScanScratch scan;
    __shared__ uint32_t found[3];
    const int tid = threadIdx.x;
    for (int b = tid * 4; b < kBins * kWideCopies; b += kThreads * 4)
        *reinterpret_cast<uint4 *>(&hist[b]) = make_uint4(0, 0, 0, 0);
    uint32_t key[4];
    load_tile(scores, N, blockIdx.x, key);
    uint32_t prefix = 0, k = (uint32_t)K;
    if constexpr (PASS > 0) wide_pick<PASS>(ws, K, pickbuf, scan, found, prefix, k);
    __syncthreads();  // the cleared histogram
    const int shift = wide_shift(PASS), shift_prev = PASS > 0 ? wide_shift(PASS - 1) : 32;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        hist_add<kWideCopies>(hist, (key[u] >> shift) & wide_mask(PASS),
                              key[u] != 0 && (PASS == 0 || (key[u] >> shift_prev) == (prefix >> shift_prev)));
    __syncthreads();
    for (int b = tid; b < kBins; b += kThreads) {
        const uint4 c = *reinterpret_cast<const uint4 *>(&hist[b * kWideCopies]);
        const uint32_t n = c.x + c.y + c.z + c.w;
        if (n) atomicAdd(&ws->ghist[PASS][b], n);
    }
}

// Picks the last digit: the threshold key and how many keys equal to it survive; counts the tile's
// keys above and equal to the threshold.
__global__ __launch_bounds__(kThreads) void topk_wide_count_kernel(const float *__restrict__ scores, int N, int K,
                                                                     WideWs *ws) {
    __shared__ uint32_t pickbuf[kBins];
    __shared__ ScanScratch scan;
    __shared__ uint32_t found[3];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint32_t key[4];
    load_tile(scores, N, blockIdx.x, key);
    uint32_t thresh, keep_eq;
    wide_pick<3>(ws, K, pickbuf, scan, found, thresh, keep_eq);
    uint32_t cnt = 0;  // low 16 bits: keys > thresh, high 16 bits: keys == thresh
#pragma unroll
    for (int u = 0; u < 4; ++u) cnt += (key[u] > thresh ? 1u : 0u) + (key[u] == thresh ? 0x10000u : 0u);
    const uint32_t inc = wave_inclusive_scan(cnt);
    if (lane == kWave - 1) scan.sums[0][wave] = inc;
    finish_scans(scan);
    if (tid == 0) {
        const uint32_t total = scan.base[0][kWaves];
        ws->counts[blockIdx.x][0] = total & 0xFFFFu;
        ws->counts[blockIdx.x][1] = total >> 16;
    }
}

// Ordered write-out of one tile; the tiles before it are accounted for by their counts.
__global__ __launch_bounds__(kThreads) void topk_wide_emit_kernel(const float *__restrict__ scores, int N,
                                                                    const WideWs *__restrict__ ws,
                                                                    int32_t *__restrict__ idx) {
    __shared__ ScanScratch scan;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint32_t key[4];
    load_tile(scores, N, blockIdx.x, key);
    const uint32_t thresh = ws->state[2][0], keep_eq = ws->state[2][1];
    uint32_t out_base = 0, eq_base = 0;  // survivors / duplicates of thresh in the tiles before this one
    for (int g = 0; g < (int)blockIdx.x; ++g) {  // uniform, at most kWideMax - 1 trips of two cached loads
        const uint32_t gt = ws->counts[g][0], eq = ws->counts[g][1];
        out_base += gt + (min(eq_base + eq, keep_eq) - min(eq_base, keep_eq));
        eq_base += eq;
    }
    uint32_t cnt = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) cnt += (key[u] > thresh ? 1u : 0u) + (key[u] == thresh ? 0x10000u : 0u);
    const uint32_t inc = wave_inclusive_scan(cnt);
    if (lane == kWave - 1) scan.sums[0][wave] = inc;
    finish_scans(scan);
    const uint32_t ex = scan.base[0][wave] + inc - cnt;
    const int i0 = blockIdx.x * kTile + tid * 4;
    uint32_t gt_before = ex & 0xFFFFu, eq_before = eq_base + (ex >> 16);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const bool gt = key[u] > thresh, eq = key[u] == thresh;
        if (gt || (eq && eq_before < keep_eq)) {
            const uint32_t eq_kept = min(eq_before, keep_eq) - min(eq_base, keep_eq);
            idx[out_base + gt_before + eq_kept] = i0 + u;
        }
        gt_before += gt ? 1u : 0u;
        eq_before += eq ? 1u : 0u;
    }
}

}  // namespace

size_t select_topk_ws(int N) {
    return (N > 8 * kTile && N <= kWideMax * kTile) ? align_up(sizeof(WideWs), 256) : 0;
}

int select_topk_varlen_max_n() { return 8 * kTile; }

int select_topk_varlen_launch(const float *scores, int ld, const SeqTab &tab, int nseq, int max_n, int32_t *idx,
                              hipStream_t s) {
    const size_t smem = (size_t)kBins * kCopies * sizeof(uint32_t);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<2, SeqTab>), smem) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<8, SeqTab>), smem))
        return STRD_EHIP;
    if (max_n <= 2 * kTile)
        select_topk_kernel<2, SeqTab><<<nseq, kThreads, smem, s>>>(scores, 0, 0, idx, tab, ld);
    else
        select_topk_kernel<8, SeqTab><<<nseq, kThreads, smem, s>>>(scores, 0, 0, idx, tab, ld);
    return launch_status();
}

int select_topk_launch(const float *scores, int N, int K, int32_t *idx, void *ws, hipStream_t s) {
    if (select_topk_ws(N)) {
        WideWs *w = reinterpret_cast<WideWs *>(ws);
        const int G = ceil_div(N, kTile);
        topk_wide_zero_kernel<<<1, kThreads, 0, s>>>(w);
        topk_wide_hist_kernel<0><<<G, kThreads, 0, s>>>(scores, N, K, w);
        topk_wide_hist_kernel<1><<<G, kThreads, 0, s>>>(scores, N, K, w);
        topk_wide_hist_kernel<2><<<G, kThreads, 0, s>>>(scores, N, K, w);
        topk_wide_count_kernel<<<G, kThreads, 0, s>>>(scores, N, K, w);
        topk_wide_emit_kernel<<<G, kThreads, 0, s>>>(scores, N, w, idx);
        return launch_status();
    }
    const size_t smem = (size_t)kBins * kCopies * sizeof(uint32_t);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<2>), smem) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<8>), smem) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<0>), smem))
        return STRD_EHIP;
    if (N <= 2 * kTile)
        select_topk_kernel<2><<<1, kThreads, smem, s>>>(scores, N, K, idx, OneSeq(), 0);
    else if (N <= 8 * kTile)
        select_topk_kernel<8><<<1, kThreads, smem, s>>>(scores, N, K, idx, OneSeq(), 0);
    else
        select_topk_kernel<0><<<1, kThreads, smem, s>>>(scores, N, K, idx, OneSeq(), 0);
    return launch_status();
}

// ---- the same selection for callers that cannot allocate --------------------------------------
// The histograms and per-tile counts of the many-workgroup form live in an array that is part of
// the library's image instead of a caller-provided workspace: every GPU the library runs on
// holds its own copy at its own address for the life of the process.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns
// for the current device.
constexpr int kStaticMaxN = kWideMax * kTile;   // 2^20 scores
constexpr size_t kStaticBytes = (sizeof(WideWs) + 255) / 256 * 256;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticBytes];

int select_topk_static_max_n() { return kStaticMaxN; }

int select_topk_static_launch(const float *scores, int N, int K, int32_t *idx, hipStream_t s) {
    constexpr int kMaxDev = 64;
    static std::mutex mu;
    static void *ptr[kMaxDev];   // device address of `scratch` on each GPU, looked up once
    if (N > kStaticMaxN || select_topk_ws(N) > kStaticBytes) return STRD_EUNSUPPORTED;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return STRD_EHIP;
    void *p = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!ptr[dev]) {
            void *q = nullptr;
            if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) {
                (void)hipGetLastError();
                return STRD_EHIP;
            }
            ptr[dev] = q;
        }
        p = ptr[dev];
    }
    // every launch of the chain starts from a kernel that clears the histograms; the counts and
    // picked digits are written before they are read
    return select_topk_launch(scores, N, K, idx, p, s);
}

}  // namespace strd
