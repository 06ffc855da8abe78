// score_mamba on bf16 matrix cores: Decoupled Content Alignment (paper Eq. "ssm_importance")
//     s_i = 1/(M*H) * sum_g (sum_{h in g} dt_i^h) * sum_m | b_i^g . c_m^g |
// The |b.c| table is an [M x N] contraction over the state dimension per group, which is never
// materialised: a wave keeps the b fragments of its 32*CT vision tokens in registers (B operand,
// tokens on the accumulator columns), streams the text rows c_m of the group through LDS as the
// A operand, and folds |acc| into one running sum per lane, so the reduction over text rows
// costs no cross-lane traffic until a single lane-half exchange at the end.
//
// Two kernels make the group partials a[g][i].
// Short sequences: one workgroup = 4 waves = 128*CT consecutive tokens of ONE group (grid = token
// tiles x groups, so even 8192 tokens give 512 workgroups); the text tile (128 rows) is
// double-buffered in LDS, filled by asynchronous global -> LDS copies, shared by the 4 waves.
// It writes a[g][i] = sum_m |b_i^g . c_m^g|, and 16 lanes per token then sum dt_i^h * a[g(h)][i]
// over the heads and scale.
// Long sequences: one workgroup per CU keeps all text rows of its group in LDS and its 8 waves
// walk a slice of the tokens with no barriers (score_mamba_res_kernel below); the dt sum of the
// group is folded in there, and a small kernel adds the groups and scales.
// No atomics, fixed summation order: bit-reproducible.  HBM traffic is one pass over B_vis and
// dt_vis; C_txt (M*n*2 bytes per group) is re-read per workgroup from L2.
// With Gaussian operands the products run at about half the nominal matrix-core rate on this
// part whatever feeds them (the same loop on register-resident random operands, with no loads
// at all, takes as long; on low-entropy operands it takes half as long): the clock under
// full-rate products of random data is what bounds the long-sequence kernel, not its loads.
#include <algorithm>

#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kMC = 128;  // text rows per LDS tile

template <int NS>
struct Tile {
    using A = AsyncTile<kMC, NS / 8, kThreads / kWave>;
    static constexpr int kPitch = A::kPitch;  // bf16 elements per LDS row
    struct alignas(16) Buf {
        bf16_t e[A::kBytes / 2];
        __device__ __forceinline__ const bf16_t *at(int r, int c) const { return e + r * kPitch + c; }
    };
    Buf c[2];
};

// FULL (the Full Mamba Dynamic score, |w_{t,j}| of paper Eq. "ssm_weight", Sec. "Why the Full Mamba Dynamic Fails"): every |b_i . c_m| is
// weighted by sum_{h in g} u_i^h v_m^h, u_i^h = dt_i^h * decay from token i to the last vision
// token, v_m^h = decay from there to text row m (both <= dt resp. 1, made by the prep kernels).
// That weight table is itself a [text row x token] contraction over the <= 16 heads of the group,
// in the accumulator layout of G^T, so it is one more MFMA per tile; u and v are split into
// bf16 high and low parts (three products) to keep about 16 bits of them.
// SEQ = SeqTab (packed batch, blockIdx.z = sequence): Bv and Ct point at the packed b and c tensors,
// the sequence's partials start at part + row0 * G.
template <int NS, int CT, bool FULL, class SEQ = OneSeq>
__global__ __launch_bounds__(kThreads) void score_mamba_mfma_kernel(const bf16_t *__restrict__ Bv,
                                                                    const bf16_t *__restrict__ Ct,
                                                                    const float *__restrict__ U,
                                                                    const float *__restrict__ V,
                                                                    float *__restrict__ part, int M, int N, int G,
                                                                    int H, SEQ seq) {
    constexpr int KS = NS / 16;  // k-steps of v_mfma_f32_32x32x16_bf16
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Tile<NS> &lds = *reinterpret_cast<Tile<NS> *>(smem_raw);
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.z;
        N = seq.N[b];
        M = seq.M[b];
        if ((int)blockIdx.x * (128 * CT) >= N) return;  // uniform: a shorter sequence than the grid was sized for
        Bv += (size_t)seq.row0[b] * G * NS;
        Ct += (size_t)(seq.row0[b] + N) * G * NS;
        part += (size_t)seq.row0[b] * G;
    }

    const int tid = threadIdx.x, lane = tid & 63, lc = lane & 31, half = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, in a scalar register
    const int g = blockIdx.y;
    const int nmc = (M + kMC - 1) / kMC;
    const int tok0 = blockIdx.x * (128 * CT) + w * (32 * CT);

    // text tiles go global -> LDS directly; rows past M re-read the last row and are skipped
    // (whole 32-row tiles) or masked (the ragged tile) when the products are folded
    using AT = typename Tile<NS>::A;
    int st_row[AT::kIssues], st_col[AT::kIssues];
#pragma unroll
    for (int i = 0; i < AT::kIssues; ++i) AT::slot(w, lane, i, st_row[i], st_col[i]);
    auto stage = [&](int mc, int b) {
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            const int m = min(mc * kMC + st_row[i], M - 1);
            AT::issue(Ct + ((size_t)m * G + g) * NS + st_col[i] * 8, &lds.c[b], w, i);
        }
    };
    stage(0, 0);

    // b fragments of this wave's tokens: lane = token column, 8 consecutive k (tail lanes repeat the last token)
    bf16x8 bfr[CT][KS];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const bf16_t *bp = Bv + ((size_t)min(tok0 + 32 * ct + lc, N - 1) * G + g) * NS + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bfr[ct][ks] = *reinterpret_cast<const bf16x8 *>(bp + 16 * ks);
    }
    // u fragments of this wave's tokens (B operand: lane = token column, k = head 8*half + j of the group)
    const int hpg = FULL ? H / G : 0;
    bf16x8 u_hi[CT], u_lo[CT];
    if (FULL) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const float *up = U + (size_t)min(tok0 + 32 * ct + lc, N - 1) * H + g * hpg + 8 * half;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float u = (8 * half + j < hpg) ? up[j] : 0.f;
                u_hi[ct][j] = (bf16_t)u;
                u_lo[ct][j] = (bf16_t)(u - (float)u_hi[ct][j]);
            }
        }
    }
    async_tile_wait();
    __syncthreads();

    float part_sum[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) part_sum[ct] = 0.f;

    for (int mc = 0; mc < nmc; ++mc) {
        const int cur = mc & 1;
        if (mc + 1 < nmc) stage(mc + 1, cur ^ 1);  // uniform
        const int mrows = M - mc * kMC;            // valid text rows of this tile (may exceed kMC)
#pragma unroll
        for (int mt = 0; mt < kMC / 32; ++mt) {
            if (32 * mt >= mrows) continue;  // uniform: tile wholly past the last text row
            f32x16 acc[CT];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[ct][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(lds.c[cur].at(32 * mt + lc, 16 * ks + 8 * half));
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfr[ct][ks], acc[ct], 0, 0, 0);
            }
            if (FULL) {
                // v fragment of the tile's text rows (A operand: lane = text row, k = head); rows past M give 0
                const int m = mc * kMC + 32 * mt + lc;
                const float *vp = V + (size_t)min(m, M - 1) * H + g * hpg + 8 * half;
                bf16x8 v_hi, v_lo;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float v = (m < M && 8 * half + j < hpg) ? vp[j] : 0.f;
                    v_hi[j] = (bf16_t)v;
                    v_lo[j] = (bf16_t)(v - (float)v_hi[j]);
                }
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    f32x16 wt;
#pragma unroll
                    for (int i = 0; i < 16; ++i) wt[i] = 0.f;
                    wt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_lo, u_hi[ct], wt, 0, 0, 0);
                    wt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, u_lo[ct], wt, 0, 0, 0);
                    wt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, u_hi[ct], wt, 0, 0, 0);
                    float t = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) t = fmaf(fabsf(acc[ct][i]), wt[i], t);
                    part_sum[ct] += t;
                }
                continue;
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                float t = 0.f;
                if (32 * mt + 32 <= mrows) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) t += fabsf(acc[ct][i]);
                } else {  // ragged tile: accumulator row i of this lane is text row 8*(i/4) + 4*half + i%4
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        t += (32 * mt + 8 * (i / 4) + 4 * half + (i % 4) < mrows) ? fabsf(acc[ct][i]) : 0.f;
                }
                part_sum[ct] += t;
            }
        }
        async_tile_wait();
        __syncthreads();
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const float col = part_sum[ct] + __shfl_xor(part_sum[ct], 32, kWave);
        const int t = tok0 + 32 * ct + lc;
        if (half == 0 && t < N) part[(size_t)g * N + t] = col;
    }
}

// s_i = 1/(M*H) * sum_h dt_i^h * a[g(h)][i].  16 adjacent lanes share a token and read its dt
// row in 64-byte pieces (coalesced); their partial sums meet in a fixed butterfly order.
template <class SEQ = OneSeq>
__global__ __launch_bounds__(kThreads) void score_mamba_reduce_kernel(const float *__restrict__ part,
                                                                      const float *__restrict__ dtv,
                                                                      float *__restrict__ s, int N, int H, int G,
                                                                      float norm, SEQ seq, int ld) {
    if constexpr (is_varlen<SEQ>()) {  // blockIdx.y = sequence; dtv is the packed tensor, s has `ld` floats per sequence
        const int b = blockIdx.y;
        N = seq.N[b];
        norm = 1.f / ((float)seq.M[b] * (float)H);
        part += (size_t)seq.row0[b] * G;
        dtv += (size_t)seq.row0[b] * H;
        s += (size_t)b * ld;
    }
    const int i = blockIdx.x * (kThreads / 16) + threadIdx.x / 16, j = threadIdx.x & 15;
    const int hpg = H / G;
    float tot = 0.f;
    if (i < N) {
        const float *dr = dtv + (size_t)i * H;
        for (int h = j; h < H; h += 16) tot = fmaf(dr[h], part[(size_t)(h / hpg) * N + i], tot);
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) tot += __shfl_xor(tot, o, kWave);
    if (i < N && j == 0) s[i] = tot * norm;
}

// Full score: the per-token factors are already inside the group partials.
__global__ __launch_bounds__(kThreads) void score_mamba_full_reduce_kernel(const float *__restrict__ part,
                                                                           float *__restrict__ s, int N, int G,
                                                                           float norm) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    float tot = 0.f;
    for (int g = 0; g < G; ++g) tot += part[(size_t)g * N + i];
    s[i] = tot * norm;
}

// ---- long sequences: the text rows of a group stay resident in LDS ------------------------------
// One workgroup = 8 waves = one group x one slice of the vision tokens (grid = slices x groups,
// at most one workgroup per CU).  The group's text rows are copied into LDS once (up to
// kResBytes of them at a time), after which the waves share nothing: each takes token tiles of
// 32*CT tokens in turn, loads their b fragments and the group's dt values straight from global
// memory, and runs through all text rows with no barrier.  Products are v_mfma_f32_16x16x32_bf16
// (A = 16 text rows, B = 16 tokens; on this chip the small form of the instruction sustains a higher
// rate than 32x32x16 at the same flops), one row tile at a time against every token tile of the wave:
// independent accumulator chains, and while they run the accumulators of the row tile before are
// folded, so the |acc| additions sit under the matrix-core work.  It writes
// a[g][i] = (sum_{h in g} dt_i^h) * sum_m |b_i^g . c_m^g|; the sum over groups and the scale are a
// second, small kernel.  The workgroups of one slice are dealt to one XCD, so that the dt rows
// (each group reads its own 4*H/G bytes of every row) meet in one L2.
typedef int strd_i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kResThreads = 512;
constexpr int kResBytes = 156 * 1024;  // LDS for text rows (160 KB per CU less a little for the runtime)
constexpr int kResPad = 2;             // pad vectors per text row: pitch = 8 words mod 32, the fast one for 16 rows x 4 pieces

template <int NS>
constexpr int res_max_rows() { return kResBytes / ((NS / 8 + kResPad) * 16) / 32 * 32; }

template <int NS, int CT>
__global__ __launch_bounds__(kResThreads) void score_mamba_res_kernel(const bf16_t *__restrict__ Bv,
                                                                      const bf16_t *__restrict__ Ct,
                                                                      const float *__restrict__ dtv,
                                                                      float *__restrict__ part, int M, int N, int G,
                                                                      int H, int slices, int slice_len) {
    constexpr int KS = NS / 32, NT = 2 * CT;  // k-steps of a product; 16-token tiles per wave tile
    constexpr int VR = NS / 8, VP = VR + kResPad, kPitch = VP * 8, kRows = res_max_rows<NS>();
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const bf16_t *text = reinterpret_cast<const bf16_t *>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, lr = lane & 15, lb = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    int slice, g;
    if (slices % kXcd == 0) {  // workgroup b runs on XCD b % 8: keep the groups of a slice together
        const int j = blockIdx.x / kXcd;
        g = j % G;
        slice = (blockIdx.x % kXcd) * (slices / kXcd) + j / G;
    } else {
        g = blockIdx.x % G;
        slice = blockIdx.x / G;
    }
    const int t_begin = slice * slice_len, t_end = min(N, t_begin + slice_len);
    const int ntile = (t_end - t_begin + 32 * CT - 1) / (32 * CT);
    const int hpg = H / G;

    for (int m0 = 0; m0 < M; m0 += kRows) {
        const int rows = min(kRows, M - m0);  // valid text rows of this pass
        const int nmt = (rows + 31) / 32;  // blocks of 32 text rows
        if (m0 > 0) __syncthreads();  // every wave is done with the previous rows
        // rows past the last one are zeros, so their products add nothing
        const int slots = nmt * 32 * VP;
        for (int s0 = w * 64; s0 < slots; s0 += (kResThreads / kWave) * 64) {
            const int s = s0 + lane, r = s / VP, cv = s % VP;
            if (s < slots && cv < VR) {
                if (r < rows)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(Ct + ((size_t)(m0 + r) * G + g) * NS + cv * 8),
                        (__attribute__((address_space(3))) void *)(smem_raw + (size_t)s0 * 16), 16, 0, 0);
                else
                    *reinterpret_cast<strd_i32x4 *>(smem_raw + (size_t)s * 16) = strd_i32x4{0, 0, 0, 0};
            }
        }
        async_tile_wait();
        __syncthreads();

        // b fragments of a wave tile: B operand, column = token lr of a 16-token tile, k slots 32 ks + 8 lb ..
        // (lanes past the end repeat the last token)
        auto load_b = [&](int tt, bf16x8(&bf)[NT][KS]) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int t = min(t_begin + tt * (32 * CT) + 16 * nt + lr, N - 1);
                const bf16_t *bp = Bv + ((size_t)t * G + g) * NS + 8 * lb;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) bf[nt][ks] = *reinterpret_cast<const bf16x8 *>(bp + 32 * ks);
            }
        };
        bf16x8 bfr[NT][KS];
        load_b(w, bfr);
        // last pass: the dt values of the group; each lane group sums a quarter of them.  With 16 heads per
        // group (rows of 16*G floats from a 16-byte aligned base: float4 loads) the values of a tile are
        // requested a whole tile before they are used: those of the first tile here, those of the next
        // tile where the current ones have been consumed.
        const bool last = m0 + kRows >= M;
        const bool dt16 = hpg == 16;
        float4 dq[NT];
        auto load_dt = [&](int tt) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                dq[nt] = *reinterpret_cast<const float4 *>(
                    dtv + (size_t)min(t_begin + tt * (32 * CT) + 16 * nt + lr, N - 1) * H + g * 16 + lb * 4);
        };
        if (last && dt16) load_dt(w);
        for (int tt = w; tt < ntile; tt += kResThreads / kWave) {
            const int tok0 = t_begin + tt * (32 * CT);
            // the fragments of this wave's next tile are requested now and used after this tile's
            // products (past the last tile they re-read the sequence's last token and are dropped)
            bf16x8 bnx[NT][KS];
            load_b(tt + kResThreads / kWave, bnx);
            // Per 16 text rows (one row tile): its products with every token tile, k-step by k-step, four
            // independent accumulator chains; meanwhile the accumulators of the row tile before are folded.
            // Each piece of a text row is replaced by the piece of the row 32 further on right after its
            // last product, a whole round of the other row tile's products before it is needed again.
            float part_sum[NT];
            f32x4 acc[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                part_sum[nt] = 0.f;
                acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // A operand: row = text row lr of a 16-row tile, k slots 32 ks + 8 lb ..
            const bf16_t *ap = text + lr * kPitch + 8 * lb;
            bf16x8 a[2][KS];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) a[rt][ks] = *reinterpret_cast<const bf16x8 *>(ap + 16 * rt * kPitch + 32 * ks);
            auto fold = [&]() {  // the accumulators of a row tile whose products are complete (zeros the first time)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    part_sum[nt] += (fabsf(acc[nt][0]) + fabsf(acc[nt][1])) + (fabsf(acc[nt][2]) + fabsf(acc[nt][3]));
            };
            // (four blocks of 32 text rows per trip: at the head of the loop the compiler waits for every LDS read
            // of the trip before, the last of which has only just been requested -- a quarter as many such waits)
            auto rows32 = [&](int mt) __attribute__((always_inline)) {
                const bf16_t *np = ap + (size_t)min(mt + 1, nmt - 1) * 32 * kPitch;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    f32x4 c[NT];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) c[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            c[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rt][ks], bfr[nt][ks], c[nt], 0, 0, 0);
                        a[rt][ks] = *reinterpret_cast<const bf16x8 *>(np + 16 * rt * kPitch + 32 * ks);
                    }
                    fold();
#pragma unroll
                    for (int i = 0; i < NT * KS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (i % NT == NT - 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                    }
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[nt] = c[nt];
                }
            };
            for (int mt = 0; mt < nmt; mt += 4) {
                rows32(mt);
                if (mt + 1 < nmt) rows32(mt + 1);  // uniform
                if (mt + 2 < nmt) rows32(mt + 2);
                if (mt + 3 < nmt) rows32(mt + 3);
            }
            fold();
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) bfr[nt][ks] = bnx[nt][ks];
            float dsum[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                dsum[nt] = 0.f;
                if (last) {
                    if (dt16) {
                        dsum[nt] = (dq[nt].x + dq[nt].y) + (dq[nt].z + dq[nt].w);
                    } else {
                        const float *dp = dtv + (size_t)min(tok0 + 16 * nt + lr, N - 1) * H + g * hpg;
                        for (int j = lb; j < hpg; j += 4) dsum[nt] += dp[j];
                    }
                }
            }
            if (last && dt16) load_dt(tt + kResThreads / kWave);  // (past the last tile: the last token again, dropped)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                // the four lane groups hold different text rows of the same token
                float col = part_sum[nt] + __shfl_xor(part_sum[nt], 16, kWave);
                col += __shfl_xor(col, 32, kWave);
                const int t = tok0 + 16 * nt + lr;
                float *dst = part + (size_t)g * N + t;
                const bool mine = lb == 0 && t < t_end;
                if (m0 > 0 && mine) col += *dst;
                if (last) {
                    float a = dsum[nt] + __shfl_xor(dsum[nt], 16, kWave);
                    a += __shfl_xor(a, 32, kWave);
                    col *= a;
                }
                if (mine) *dst = col;
            }
        }
    }
}

// Token slices of the resident-text kernel: as many as fill the CUs, a multiple of 8 when
// possible (XCD placement), each a whole number of 32*CT-token tiles.
inline void res_plan(int N, int G, int ct, int *slices, int *slice_len) {
    int want = std::max(1, 256 / G);
    if (want >= kXcd) want = want / kXcd * kXcd;
    const int tile = 32 * ct;
    int len = (ceil_div(N, want) + tile - 1) / tile * tile;
    int ns = ceil_div(N, len);
    if (ns >= kXcd && ns % kXcd) {  // a little shorter slices so that their number is a multiple of 8 again
        const int up = (ns + kXcd - 1) / kXcd * kXcd;
        const int len2 = (ceil_div(N, up) + tile - 1) / tile * tile;
        if (ceil_div(N, len2) % kXcd == 0) { len = len2; ns = ceil_div(N, len2); }
    }
    *slices = ns;
    *slice_len = len;
}

template <int NS, int CT>
int launch_res(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, void *ws,
               hipStream_t st) {
    const int rows = std::min(res_max_rows<NS>(), (M + 31) / 32 * 32);
    const size_t smem = (size_t)rows * (NS / 8 + kResPad) * 16;
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&score_mamba_res_kernel<NS, CT>), smem)) return STRD_EHIP;
    int slices, slice_len;
    res_plan(N, G, CT, &slices, &slice_len);
    float *part = (float *)ws;
    score_mamba_res_kernel<NS, CT><<<slices * G, kResThreads, smem, st>>>((const bf16_t *)B, (const bf16_t *)C, dt, part,
                                                                         M, N, G, H, slices, slice_len);
    score_mamba_full_reduce_kernel<<<ceil_div(N, kThreads), kThreads, 0, st>>>(part, s, N, G,
                                                                             1.f / ((float)M * (float)H));
    return launch_status();
}

template <int NS, int CT>
int launch_full(const void *B, const void *C, const float *U, const float *V, float *s, int M, int N, int H, int G,
                void *ws, hipStream_t st) {
    const size_t smem = sizeof(Tile<NS>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&score_mamba_mfma_kernel<NS, CT, true>), smem))
        return STRD_EHIP;
    float *part = (float *)ws;
    const dim3 grid(ceil_div(N, 128 * CT), G);
    score_mamba_mfma_kernel<NS, CT, true><<<grid, kThreads, smem, st>>>((const bf16_t *)B, (const bf16_t *)C, U, V, part,
                                                                        M, N, G, H, OneSeq());
    score_mamba_full_reduce_kernel<<<ceil_div(N, kThreads), kThreads, 0, st>>>(part, s, N, G,
                                                                             1.f / ((float)M * (float)H));
    return launch_status();
}

template <int NS, int CT>
int launch(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, void *ws,
           hipStream_t st) {
    const size_t smem = sizeof(Tile<NS>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&score_mamba_mfma_kernel<NS, CT, false>), smem))
        return STRD_EHIP;
    float *part = (float *)ws;
    const dim3 grid(ceil_div(N, 128 * CT), G);
    score_mamba_mfma_kernel<NS, CT, false><<<grid, kThreads, smem, st>>>((const bf16_t *)B, (const bf16_t *)C, nullptr,
                                                                         nullptr, part, M, N, G, H, OneSeq());
    score_mamba_reduce_kernel<<<ceil_div(N, kThreads / 16), kThreads, 0, st>>>(part, dt, s, N, H, G,
                                                                          1.f / ((float)M * (float)H), OneSeq(), 0);
    return launch_status();
}

template <int NS>
int launch_varlen(const void *B, const void *C, const float *dt, float *s, int ld, const SeqTab &tab, int nseq, int max_n, int H, int G,
                  void *ws, hipStream_t st) {
    const size_t smem = sizeof(Tile<NS>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&score_mamba_mfma_kernel<NS, 1, false, SeqTab>), smem))
        return STRD_EHIP;
    float *part = (float *)ws;
    score_mamba_mfma_kernel<NS, 1, false, SeqTab><<<dim3(ceil_div(max_n, 128), G, nseq), kThreads, smem, st>>>(
        (const bf16_t *)B, (const bf16_t *)C, nullptr, nullptr, part, 0, 0, G, H, tab);
    score_mamba_reduce_kernel<SeqTab><<<dim3(ceil_div(max_n, kThreads / 16), nseq), kThreads, 0, st>>>(part, dt, s, 0, H, G,
                                                                                               0.f, tab, ld);
    return launch_status();
}

}  // namespace

// Packed batch on the matrix-core tile kernel: partials of sequence b at ws + row0[b] * G floats.
int score_mamba_mfma_varlen(const void *B, const void *C, const float *dt, float *s, int ld, const SeqTab &tab, int nseq, int max_n,
                            int H, int G, int n, void *ws, hipStream_t st) {
    if (n == 128) return launch_varlen<128>(B, C, dt, s, ld, tab, nseq, max_n, H, G, ws, st);
    if (n == 64) return launch_varlen<64>(B, C, dt, s, ld, tab, nseq, max_n, H, G, ws, st);
    return STRD_EUNSUPPORTED;
}

bool score_mamba_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io) {
    (void)M; (void)H;
    return io == STRD_BF16 && (n == 64 || n == 128) && N >= 1 && G <= 65535;
}

size_t score_mamba_mfma_ws(int N, int G) { return align_up((size_t)G * N * sizeof(float), 256); }

int score_mamba_mfma(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, int n,
                     void *ws, hipStream_t st) {
    // Long sequences: text rows resident in LDS, one workgroup per CU.  It pays once every wave
    // has a few token tiles of its own (one slice = N / (256 / G) tokens, shared by 8 waves).
    // (Wave tiles of 32 tokens: with 64 the kernel is no faster and, at n = 128, out of registers.)
    const long long per_slice = (long long)N / std::max(1, 256 / G);
    if (per_slice >= 512)
        return n == 128 ? launch_res<128, 1>(B, C, dt, s, M, N, H, G, ws, st) : launch_res<64, 1>(B, C, dt, s, M, N, H, G, ws, st);
    // wide token tiles once there are enough of them to fill 256 CUs several times over
    const bool wide = (long long)N * G >= 256LL * 256 * 8;
    if (n == 128)
        return wide ? launch<128, 2>(B, C, dt, s, M, N, H, G, ws, st) : launch<128, 1>(B, C, dt, s, M, N, H, G, ws, st);
    if (n == 64)
        return wide ? launch<64, 2>(B, C, dt, s, M, N, H, G, ws, st) : launch<64, 1>(B, C, dt, s, M, N, H, G, ws, st);
    return STRD_EUNSUPPORTED;
}

// Full score on matrix cores: needs the heads of a group to fit one k = 16 product.
bool score_mamba_full_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io) {
    return score_mamba_mfma_supported(M, N, H, G, n, io) && H / G <= 16;
}

int score_mamba_full_mfma(const void *B, const void *C, const float *U, const float *V, float *s, int M, int N, int H,
                          int G, int n, void *part_ws, hipStream_t st) {
    if (n == 128) return launch_full<128, 1>(B, C, U, V, s, M, N, H, G, part_ws, st);
    if (n == 64) return launch_full<64, 1>(B, C, U, V, s, M, N, H, G, part_ws, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
