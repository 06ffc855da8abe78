// score_attn on bf16 matrix cores: text-to-vision attention importance (paper Sec. 3.1,
// "Attention Layers")
//     s_i = 1/(M*Hq) * sum_{m,h} softmax_i( scale * q_m^h . k_i^{kv(h)} ),  softmax over the N keys.
// The [M*Hq x N] probability table is never stored; it is produced twice, tile by tile:
//   pass 1 (stats)   per query row: running max and sum of 2^z over a slice of the keys,
//   combine          per query row: log2-sum-exp over the slices,
//   pass 2 (colsum)  per key: sum over the query rows of 2^(z - lse),
//   reduce           sum over kv heads, times 1/(M*Hq).
// with z = q.k * scale * log2(e).  Both passes compute the tile transposed, Z^T[key, query]
// (A operand = key rows, B operand = query rows, v_mfma_f32_32x32x16_bf16), so a lane holds one
// query column and 16 keys: the per-query softmax state of pass 1 and the per-query lse of
// pass 2 are one scalar per lane.  In pass 1 a wave keeps its query fragments in registers and
// streams keys through LDS; in pass 2 a wave keeps its key fragments in registers, streams the
// query rows of its kv head through LDS and accumulates 2^(z-lse) per (lane, key) over all
// query tiles before a single butterfly reduction over the 32 lanes.  All reductions run in a
// fixed order: the scores are bit-reproducible.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kRows = 128;  // rows (keys in pass 1, queries in pass 2) per LDS tile
constexpr int kTW = 2;      // 32-wide register tiles per wave (queries in pass 1, keys in pass 2)
constexpr float kLog2e = 1.4426950408889634f;

template <int D>
struct Tile {
    using A = AsyncTile<kRows, D / 8, kThreads / kWave>;
    static constexpr int kPitch = A::kPitch;
    struct alignas(16) Buf {
        bf16_t e[A::kBytes / 2];
        __device__ __forceinline__ const bf16_t *at(int r, int c) const { return e + r * kPitch + c; }
    };
    Buf t[2];
    float lse[2][kRows];
};

__device__ __forceinline__ float ex2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 zero16() {
    f32x16 v;
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = 0.f;
    return v;
}

// Query row r of kv head kvh (r = m * rep + j) lives at q[(m * Hq + kvh * rep + j) * D].
__device__ __forceinline__ size_t qrow_index(int r, int rep, int Hq, int kvh) {
    return (size_t)(r / rep) * Hq + kvh * rep + r % rep;
}

// ---------------------------------------------------------------------------------------------
// pass 1: grid = row blocks (fastest) x kv heads x key slices
// SEQ = SeqTab (packed batch, blockIdx.y = sequence): q and k point at the packed tensors and every
// sequence has `seq_stride` floats of pmax / psum of its own; the grid and the key slices are those of
// the longest sequence, so a shorter one leaves slices empty (max = -inf, sum = 0).
template <int D, class SEQ>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_stats_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                              float *__restrict__ pmax, float *__restrict__ psum, int M,
                                                              int N, int Hq, int Hkv, float scale2, int nrb,
                                                              int keys_per_slice, int nunits, SEQ seq, size_t seq_stride) {
    constexpr int KS = D / 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Tile<D> &lds = *reinterpret_cast<Tile<D> *>(smem_raw);
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        N = seq.N[b];
        M = seq.M[b];
        k += (size_t)seq.row0[b] * Hkv * D;
        q += (size_t)(seq.row0[b] + N) * Hq * D;
        pmax += b * seq_stride;
        psum += b * seq_stride;
    }
    const int tid = threadIdx.x, lane = tid & 63, lc = lane & 31, half = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, in a scalar register
    const int rep = Hq / Hkv, R = M * rep;
    // the row blocks of one (kv head, slice) stream the same keys: keep them on one XCD's L2
    const int unit = xcd_swizzle(blockIdx.x, nunits);
    if (unit >= nunits) return;
    const int rb = unit % nrb, kvh = (unit / nrb) % Hkv, sl = unit / (nrb * Hkv);
    const int key0 = sl * keys_per_slice, key1 = min(N, key0 + keys_per_slice);
    const int nchunk = (key1 - key0 + kRows - 1) / kRows;

    // this wave's query fragments (B operand: lane = query column)
    bf16x8 bq[kTW][KS];
    int row[kTW];
#pragma unroll
    for (int qt = 0; qt < kTW; ++qt) {
        row[qt] = rb * (4 * 32 * kTW) + w * (32 * kTW) + 32 * qt + lc;
        const bf16_t *qp = q + qrow_index(min(row[qt], R - 1), rep, Hq, kvh) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bq[qt][ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks + 8 * half);
    }

    // key tiles go global -> LDS directly; this lane's slots of a tile are fixed
    using AT = typename Tile<D>::A;
    int st_row[AT::kIssues], st_col[AT::kIssues];
#pragma unroll
    for (int i = 0; i < AT::kIssues; ++i) AT::slot(w, lane, i, st_row[i], st_col[i]);
    auto stage = [&](int chunk, int b) {
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            const int key = min(key0 + chunk * kRows + st_row[i], N - 1);
            AT::issue(k + ((size_t)key * Hkv + kvh) * D + st_col[i] * 8, &lds.t[b], w, i);
        }
    };

    float run_m[kTW], run_s[kTW];
#pragma unroll
    for (int qt = 0; qt < kTW; ++qt) { run_m[qt] = -INFINITY; run_s[qt] = 0.f; }

    stage(0, 0);
    async_tile_wait();
    __syncthreads();
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int cur = chunk & 1;
        stage(min(chunk + 1, nchunk - 1), cur ^ 1);
        const int kbase = key0 + chunk * kRows;
        // Units of work: (key tile kt, query tile qt): 8 products, then the online (max, sum) update
        // with 16 exponentials.  In a full chunk the products of the next unit are issued with the
        // vector arithmetic of the current one (two accumulators).
        auto load_k = [&](int kt, bf16x8 (&kf)[KS]) {  // all fragments of a tile at once: one LDS round trip
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[ks] = *reinterpret_cast<const bf16x8 *>(lds.t[cur].at(32 * kt + lc, 16 * ks + 8 * half));
        };
        auto products = [&](int qt, const bf16x8 (&kf)[KS]) {
            f32x16 acc = zero16();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = mfma32(kf[ks], bq[qt][ks], acc);
            return acc;
        };
        // running max in log2 units; the scale (> 0) commutes with the max and is folded into the
        // exponent's fma
        auto fold = [&](int qt, const f32x16 &acc) {
            float tmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, acc[i]);
            const float nm = fmaxf(run_m[qt], tmax * scale2);
            const float ref = (nm == -INFINITY) ? 0.f : nm;
            float ts = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) ts += ex2(fmaf(acc[i], scale2, -ref));
            run_s[qt] = run_s[qt] * ex2(run_m[qt] - ref) + ts;
            run_m[qt] = nm;
        };
        auto interleave = [] {  // per product: its share of the 16 fma / exp / add and of the 8 max3
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 24 / KS, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 16 / KS, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 16 / KS, 0);
            }
        };
        static_assert(kTW == 2, "two query tiles per wave");
        bf16x8 kf[KS];
        if (kbase + kRows <= key1) {  // uniform: every key of the chunk belongs to the slice -- one straight block
            load_k(0, kf);
            f32x16 acc0 = products(0, kf), acc1;
#pragma unroll
            for (int kt = 0; kt < kRows / 32; ++kt) {
                acc1 = products(1, kf);  // last use of this tile's fragments
                if (kt + 1 < kRows / 32) load_k(kt + 1, kf);
                fold(0, acc0);
                interleave();
                if (kt + 1 < kRows / 32) acc0 = products(0, kf);
                fold(1, acc1);
                if (kt + 1 < kRows / 32) interleave();
            }
        } else {
            for (int kt = 0; kbase + 32 * kt < key1; ++kt) {  // ragged last chunk: tile by tile, keys past the slice masked
                load_k(kt, kf);
                f32x16 acc[kTW] = {products(0, kf), products(1, kf)};
                if (kbase + 32 * kt + 32 > key1) {
#pragma unroll
                    for (int qt = 0; qt < kTW; ++qt)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            if (kbase + 32 * kt + 8 * (i / 4) + 4 * half + (i % 4) >= key1) acc[qt][i] = -INFINITY;
                }
                fold(0, acc[0]);
                fold(1, acc[1]);
            }
        }
        async_tile_wait();
        __syncthreads();
    }
    // merge the two lane halves (disjoint keys of the same query) and publish
#pragma unroll
    for (int qt = 0; qt < kTW; ++qt) {
        const float om = __shfl_xor(run_m[qt], 32, kWave), os = __shfl_xor(run_s[qt], 32, kWave);
        const float nm = fmaxf(run_m[qt], om);
        const float ref = (nm == -INFINITY) ? 0.f : nm;
        const float tot = run_s[qt] * ex2(run_m[qt] - ref) + os * ex2(om - ref);
        if (half == 0 && row[qt] < R) {
            const size_t o = (size_t)sl * M * Hq + qrow_index(row[qt], rep, Hq, kvh);
            pmax[o] = nm;
            psum[o] = tot;
        }
    }
}

// combine: lse2[row] = log2 sum over slices.  A workgroup takes 16 rows; thread (j, r) = (tid / 16,
// tid % 16) folds slices j, j + 16, ... of row r (16 adjacent rows per load: coalesced), then the 16
// partial (max, sum) pairs of a row meet in LDS in a fixed order.
template <class SEQ>
__global__ __launch_bounds__(kThreads) void attn_lse_kernel(const float *__restrict__ pmax, const float *__restrict__ psum,
                                                            float *__restrict__ lse2, int rows, int nslice, SEQ seq,
                                                            int Hq, size_t seq_stride, int lse_ld) {
    __shared__ float sm[16][17], ss[16][17];
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        rows = seq.M[b] * Hq;
        if ((int)blockIdx.x * 16 >= rows) return;  // uniform
        pmax += b * seq_stride;
        psum += b * seq_stride;
        lse2 += (size_t)b * lse_ld;
    }
    const int j = threadIdx.x >> 4, rr = threadIdx.x & 15;
    const int r = min(blockIdx.x * 16 + rr, rows - 1);
    float m = -INFINITY, tot = 0.f;
    for (int s = j; s < nslice; s += 16) {  // online (max, sum) over this thread's slices
        const float pm = pmax[(size_t)s * rows + r], ps = psum[(size_t)s * rows + r];
        if (pm != -INFINITY) {
            const float nm = fmaxf(m, pm);
            tot = tot * ex2(m - nm) + ps * ex2(pm - nm);
            m = nm;
        }
    }
    sm[j][rr] = m;
    ss[j][rr] = tot;
    __syncthreads();
    if (j == 0 && blockIdx.x * 16 + rr < rows) {
        float gm = -INFINITY;
        for (int q = 0; q < 16; ++q) gm = fmaxf(gm, sm[q][rr]);
        float t = 0.f;
        for (int q = 0; q < 16; ++q)
            if (sm[q][rr] != -INFINITY) t += ss[q][rr] * ex2(sm[q][rr] - gm);
        lse2[r] = gm + __log2f(t);
    }
}

// ---------------------------------------------------------------------------------------------
// pass 2: grid = kv heads (fastest) x key blocks
template <int D, class SEQ>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_colsum_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                               const float *__restrict__ lse2, float *__restrict__ part,
                                                               int M, int N, int Hq, int Hkv, float scale2, SEQ seq,
                                                               int lse_ld, size_t part_stride) {
    constexpr int KS = D / 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Tile<D> &lds = *reinterpret_cast<Tile<D> *>(smem_raw);
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        N = seq.N[b];
        M = seq.M[b];
        if ((int)(blockIdx.x / Hkv) * (4 * 32 * kTW) >= N) return;  // uniform: key block past this sequence's keys
        k += (size_t)seq.row0[b] * Hkv * D;
        q += (size_t)(seq.row0[b] + N) * Hq * D;
        lse2 += (size_t)b * lse_ld;
        part += b * part_stride;
    }
    const int tid = threadIdx.x, lane = tid & 63, lc = lane & 31, half = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, in a scalar register
    const int rep = Hq / Hkv, R = M * rep;
    const int kvh = blockIdx.x % Hkv, kb = blockIdx.x / Hkv;
    const int nchunk = (R + kRows - 1) / kRows;

    // this wave's key fragments (A operand: lane = key row)
    bf16x8 ak[kTW][KS];
    const int kbase = kb * (4 * 32 * kTW) + w * (32 * kTW);
#pragma unroll
    for (int kt = 0; kt < kTW; ++kt) {
        const bf16_t *kp = k + ((size_t)min(kbase + 32 * kt + lc, N - 1) * Hkv + kvh) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) ak[kt][ks] = *reinterpret_cast<const bf16x8 *>(kp + 16 * ks + 8 * half);
    }

    // query tiles go global -> LDS directly; the lse of the tile's rows goes through a register
    // (the slots of this lane are recomputed for every tile, a few integer operations, rather than
    // held in registers: the kernel needs all 256 of them for operands and accumulators)
    using AT = typename Tile<D>::A;
    float stage_lse = 0.f;
    // rows per kv head are usually a power of two: shift and mask instead of a division per copy
    const int rep_shift = (rep & (rep - 1)) == 0 ? __builtin_ctz(rep) : -1;  // uniform
    auto stage = [&](int chunk, int b) {
        int lane_now = lane;
        asm volatile("" : "+v"(lane_now));  // keeps the slot arithmetic here instead of in registers across the loop
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            int st_row, st_col;
            AT::slot(w, lane_now, i, st_row, st_col);
            const int rr = min(chunk * kRows + st_row, R - 1);
            const size_t qi = rep_shift >= 0 ? (size_t)(rr >> rep_shift) * Hq + kvh * rep + (rr & (rep - 1))
                                             : qrow_index(rr, rep, Hq, kvh);
            AT::issue(q + qi * D + st_col * 8, &lds.t[b], w, i);
        }
        if (tid < kRows) {
            const int rr = chunk * kRows + tid;
            // rows past the end get lse = +inf, so their probabilities are exactly 0
            stage_lse = (rr < R) ? lse2[qrow_index(rr, rep, Hq, kvh)] : INFINITY;
        }
    };
    auto stage_lse_store = [&](int b) {
        if (tid < kRows) lds.lse[b][tid] = stage_lse;
    };

    float col[kTW * 16];
#pragma unroll
    for (int j = 0; j < kTW * 16; ++j) col[j] = 0.f;

    stage(0, 0);
    stage_lse_store(0);
    async_tile_wait();
    __syncthreads();
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int cur = chunk & 1;
        stage(min(chunk + 1, nchunk - 1), cur ^ 1);
        // Units of work: (query tile qt, key tile kt), 8 products each, then 16 exponentials folded
        // into the column sums.  The products of the next unit are issued before the exponentials
        // of the current one (two accumulators), so the matrix pipe works while the wave does its
        // vector arithmetic.  Query tiles wholly past the end are skipped (uniform).
        auto load_q = [&](int qt, bf16x8 (&qf)[KS]) {  // all fragments of a tile at once: one LDS round trip
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qf[ks] = *reinterpret_cast<const bf16x8 *>(lds.t[cur].at(32 * qt + lc, 16 * ks + 8 * half));
        };
        auto products = [&](int kt, const bf16x8 (&qf)[KS]) {
            f32x16 acc = zero16();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = mfma32(ak[kt][ks], qf[ks], acc);
            return acc;
        };
        auto fold = [&](int kt, const f32x16 &acc, float lse) {
#pragma unroll
            for (int i = 0; i < 16; ++i) col[kt * 16 + i] += ex2(fmaf(acc[i], scale2, -lse));
        };
        // ask the scheduler for one product, then six vector instructions (2 x fma, exp, add), eight times
        auto interleave = [] {
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one product
                __builtin_amdgcn_sched_group_barrier(0x002, 16 / KS, 0);  // fma of the next elements
                __builtin_amdgcn_sched_group_barrier(0x400, 16 / KS, 0);  // their exponentials
                __builtin_amdgcn_sched_group_barrier(0x002, 16 / KS, 0);  // adds of the previous ones
            }
        };
        static_assert(kTW == 2, "two key tiles per wave");
        bf16x8 qf[KS];
        if (chunk * kRows + kRows <= R) {  // uniform: every query tile of the chunk is real -- one straight block
            load_q(0, qf);
            float lse = lds.lse[cur][lc];
            f32x16 acc0 = products(0, qf), acc1;
#pragma unroll
            for (int qt = 0; qt < kRows / 32; ++qt) {
                acc1 = products(1, qf);  // last use of this tile's fragments
                float lse_next = 0.f;
                if (qt + 1 < kRows / 32) {
                    load_q(qt + 1, qf);
                    lse_next = lds.lse[cur][32 * (qt + 1) + lc];
                }
                fold(0, acc0, lse);
                interleave();
                if (qt + 1 < kRows / 32) acc0 = products(0, qf);
                fold(1, acc1, lse);
                if (qt + 1 < kRows / 32) interleave();
                lse = lse_next;
            }
        } else {
            for (int qt = 0; chunk * kRows + 32 * qt < R; ++qt) {  // ragged last chunk: tile by tile
                load_q(qt, qf);
                const float lse = lds.lse[cur][32 * qt + lc];
                const f32x16 acc0 = products(0, qf), acc1 = products(1, qf);
                fold(0, acc0, lse);
                fold(1, acc1, lse);
            }
        }
        stage_lse_store(cur ^ 1);
        async_tile_wait();
        __syncthreads();
    }

    // butterfly over the 32 query lanes of each half: afterwards lane lc holds the total of
    // register lc (= key tile lc / 16, accumulator row lc % 16)
    static_assert(kTW == 2, "the butterfly below reduces 32 registers over 32 lanes");
#pragma unroll
    for (int step = 0; step < 5; ++step) {
        const int mask = 16 >> step, cnt = 16 >> step;
        const bool up = (lc & mask) != 0;
#pragma unroll
        for (int j = 0; j < cnt; ++j) {
            const float send = up ? col[j] : col[j + cnt];
            const float keep = up ? col[j + cnt] : col[j];
            col[j] = keep + __shfl_xor(send, mask, kWave);
        }
    }
    const int kt = lc >> 4, i = lc & 15;
    const int key = kbase + 32 * kt + 8 * (i / 4) + 4 * half + (i % 4);
    if (key < N) part[(size_t)kvh * N + key] = col[0];
}

template <class SEQ>
__global__ __launch_bounds__(kThreads) void attn_score_reduce_kernel(const float *__restrict__ part, float *__restrict__ s,
                                                                     int N, int Hkv, float norm, SEQ seq, int Hq,
                                                                     size_t part_stride, int ld) {
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        N = seq.N[b];
        norm = 1.f / ((float)seq.M[b] * (float)Hq);
        part += b * part_stride;
        s += (size_t)b * ld;
    }
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    float t = 0.f;
    for (int h = 0; h < Hkv; ++h) t += part[(size_t)h * N + i];
    s[i] = t * norm;
}

struct Plan {
    int nrb, nslice, keys_per_slice;
};

Plan make_plan(int M, int N, int Hq, int Hkv) {
    Plan p;
    const int R = M * (Hq / Hkv);
    p.nrb = ceil_div(R, 4 * 32 * kTW);
    // enough key slices to give the chip a few waves of workgroups, at least one LDS tile each
    int want = ceil_div(1024, p.nrb * Hkv);
    const int max_slices = ceil_div(N, kRows);
    if (want > max_slices) want = max_slices;
    if (want < 1) want = 1;
    p.keys_per_slice = ceil_div(ceil_div(N, want), kRows) * kRows;
    p.nslice = ceil_div(N, p.keys_per_slice);
    return p;
}

// One sequence (SEQ = OneSeq, nseq = 1) or a packed batch: M and N are then the largest text and
// vision counts of the batch, and every sequence has a plan's worth of workspace of its own.
template <int D, class SEQ>
int run(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, float scale, void *ws, const SEQ &seq,
        int nseq, int ld, hipStream_t st) {
    const Plan p = make_plan(M, N, Hq, Hkv);
    const size_t smem = sizeof(Tile<D>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&attn_stats_kernel<D, SEQ>), smem) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&attn_colsum_kernel<D, SEQ>), smem))
        return STRD_EHIP;
    // per sequence: pmax | psum | lse | part, sequence after sequence inside each of the four regions
    const size_t rows = (size_t)M * Hq;
    const size_t stat_stride = rows * p.nslice, part_stride = (size_t)Hkv * N;
    float *pmax = (float *)ws, *psum = pmax + stat_stride * nseq;
    float *lse2 = psum + stat_stride * nseq, *part = lse2 + align_up(rows * nseq, 64);
    const float scale2 = scale * kLog2e;
    const int nunits = p.nrb * Hkv * p.nslice;
    attn_stats_kernel<D, SEQ><<<dim3(xcd_grid(nunits), nseq), kThreads, smem, st>>>(
        (const bf16_t *)q, (const bf16_t *)k, pmax, psum, M, N, Hq, Hkv, scale2, p.nrb, p.keys_per_slice, nunits, seq,
        stat_stride);
    attn_lse_kernel<SEQ><<<dim3(ceil_div((int)rows, 16), nseq), kThreads, 0, st>>>(pmax, psum, lse2, (int)rows, p.nslice, seq, Hq,
                                                                                  stat_stride, (int)rows);
    const int nkb = ceil_div(N, 4 * 32 * kTW);
    attn_colsum_kernel<D, SEQ><<<dim3(nkb * Hkv, nseq), kThreads, smem, st>>>((const bf16_t *)q, (const bf16_t *)k, lse2, part,
                                                                              M, N, Hq, Hkv, scale2, seq, (int)rows,
                                                                              part_stride);
    attn_score_reduce_kernel<SEQ><<<dim3(ceil_div(N, kThreads), nseq), kThreads, 0, st>>>(
        part, s, N, Hkv, 1.f / ((float)M * (float)Hq), seq, Hq, part_stride, ld);
    return launch_status();
}

size_t ws_bytes(int M, int N, int Hq, int Hkv, int nseq) {
    const Plan p = make_plan(M, N, Hq, Hkv);
    const size_t rows = (size_t)M * Hq;
    return align_up((2 * rows * p.nslice * nseq + align_up(rows * nseq, 64) + (size_t)Hkv * N * nseq) * sizeof(float), 256);
}

}  // namespace

bool score_attn_mfma_supported(int M, int N, int Hq, int Hkv, int d, strd_dtype io) {
    if (io != STRD_BF16 || (d != 64 && d != 128)) return false;
    const long long blocks1 = (long long)ceil_div(M * (Hq / Hkv), 4 * 32 * kTW) * Hkv * ceil_div(N, kRows);
    const long long blocks2 = (long long)ceil_div(N, 4 * 32 * kTW) * Hkv;
    return blocks1 < (1LL << 30) && blocks2 < (1LL << 30) && (long long)M * Hq < (1LL << 30);
}

size_t score_attn_mfma_ws(int M, int N, int Hq, int Hkv) { return ws_bytes(M, N, Hq, Hkv, 1); }
size_t score_attn_mfma_varlen_ws(int nseq, int max_m, int max_n, int Hq, int Hkv) {
    return ws_bytes(max_m, max_n, Hq, Hkv, nseq);
}

int score_attn_mfma(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, int d, float scale, void *ws,
                    hipStream_t st) {
    if (d == 128) return run<128>(q, k, s, M, N, Hq, Hkv, scale, ws, OneSeq(), 1, 0, st);
    if (d == 64) return run<64>(q, k, s, M, N, Hq, Hkv, scale, ws, OneSeq(), 1, 0, st);
    return STRD_EUNSUPPORTED;
}

int score_attn_mfma_varlen(const void *q, const void *k, float *s, int ld, const SeqTab &tab, int nseq, int max_m,
                           int max_n, int Hq, int Hkv, int d, float scale, void *ws, hipStream_t st) {
    if (d == 128) return run<128>(q, k, s, max_m, max_n, Hq, Hkv, scale, ws, tab, nseq, ld, st);
    if (d == 64) return run<64>(q, k, s, max_m, max_n, Hq, Hkv, scale, ws, tab, nseq, ld, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
