// score_mamba on bf16 matrix cores: Decoupled Content Alignment (paper Eq. "ssm_importance")
//     s_i = 1/(M*H) * sum_g (sum_{h in g} dt_i^h) * sum_m | b_i^g . c_m^g |
// The |b.c| table is an [M x N] contraction over the state dimension per group, which is never
// materialised: a wave keeps the b fragments of its 32*CT vision tokens in registers (B operand,
// tokens on the accumulator columns), streams the text rows c_m of the group through LDS as the
// A operand, and folds |acc| into one running sum per lane, so the reduction over text rows
// costs no cross-lane traffic until the single lane-half exchange at the end of a group.  The
// sum over groups stays inside the lane, in group order: no atomics, bit-reproducible.
//
// One workgroup = 4 waves = 128*CT consecutive tokens, all groups.  The text tile (128 rows
// of one group) is double-buffered in LDS and shared by the 4 waves; the next tile and the
// next group's b fragments are prefetched (tile: asynchronous global -> LDS copy, fragments:
// registers) while the current tile is consumed.
// HBM traffic is one pass over B_vis and dt_vis; C_txt (M*G*n*2 bytes) is re-read per
// workgroup from L2.
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

template <int NS, int CT>
__global__ __launch_bounds__(kThreads) void score_mamba_mfma_kernel(const bf16_t *__restrict__ Bv,
                                                                    const bf16_t *__restrict__ Ct,
                                                                    const float *__restrict__ dtv,
                                                                    float *__restrict__ s, int M, int N, int H, int G) {
    constexpr int KS = NS / 16;  // k-steps of v_mfma_f32_32x32x16_bf16
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Tile<NS> &lds = *reinterpret_cast<Tile<NS> *>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lc = lane & 31, half = lane >> 5;
    const int hpg = H / G;
    const int nmc = (M + kMC - 1) / kMC, nchunk = G * nmc;
    const int tok0 = blockIdx.x * (128 * CT) + w * (32 * CT);
    int tok[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) tok[ct] = min(tok0 + 32 * ct + lc, N - 1);  // tail lanes repeat the last token

    // text tiles go global -> LDS directly; rows past M re-read the last row and are skipped
    // (whole 32-row tiles) or masked (the ragged tile) when the products are folded
    using AT = typename Tile<NS>::A;
    int st_row[AT::kIssues], st_col[AT::kIssues];
#pragma unroll
    for (int i = 0; i < AT::kIssues; ++i) AT::slot(w, lane, i, st_row[i], st_col[i]);
    auto stage = [&](int chunk, int b) {
        const int g = chunk / nmc, m0 = (chunk % nmc) * kMC;
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            const int m = min(m0 + st_row[i], M - 1);
            AT::issue(Ct + ((size_t)m * G + g) * NS + st_col[i] * 8, &lds.c[b], w, i);
        }
    };
    // b fragments of group g for this wave's tokens: lane = token column, 8 consecutive k
    auto load_b = [&](bf16x8 (&dst)[CT][KS], int g) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                dst[ct][ks] = *reinterpret_cast<const bf16x8 *>(Bv + ((size_t)tok[ct] * G + g) * NS + 16 * ks + 8 * half);
    };

    bf16x8 bcur[CT][KS], bnext[CT][KS];
    load_b(bcur, 0);
    stage(0, 0);
    async_tile_wait();
    __syncthreads();

    float total[CT], part[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) total[ct] = part[ct] = 0.f;

    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int g = chunk / nmc, mc = chunk % nmc, cur = chunk & 1;
        // prefetch (clamped, so the loop body is free of conditional loads)
        stage(min(chunk + 1, nchunk - 1), cur ^ 1);
        if (mc == 0) load_b(bnext, min(g + 1, G - 1));
        const int mrows = M - mc * kMC;  // valid text rows of this tile (may exceed kMC)

        // |c_m . b_i| for the 128 text rows of this tile, 32 at a time
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
                    acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bcur[ct][ks], acc[ct], 0, 0, 0);
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
                part[ct] += t;
            }
        }

        if (mc == nmc - 1) {
            // end of a group: weight by the summed dt of the group's heads
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                float dts = 0.f;
                for (int j = half; j < hpg; j += 2) dts += dtv[(size_t)tok[ct] * H + g * hpg + j];
                dts += __shfl_xor(dts, 32, kWave);
                const float col = part[ct] + __shfl_xor(part[ct], 32, kWave);
                total[ct] += dts * col;
                part[ct] = 0.f;
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) bcur[ct][ks] = bnext[ct][ks];
        }
        async_tile_wait();
        __syncthreads();
    }

    const float norm = 1.f / ((float)M * (float)H);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int t = tok0 + 32 * ct + lc;
        if (half == 0 && t < N) s[t] = total[ct] * norm;
    }
}

template <int NS, int CT>
int launch(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, hipStream_t st) {
    const size_t smem = sizeof(Tile<NS>);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&score_mamba_mfma_kernel<NS, CT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return STRD_EHIP;
        configured = true;
    }
    const int grid = ceil_div(N, 128 * CT);
    score_mamba_mfma_kernel<NS, CT><<<grid, kThreads, smem, st>>>((const bf16_t *)B, (const bf16_t *)C, dt, s, M, N, H, G);
    return launch_status();
}

}  // namespace

bool score_mamba_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io) {
    (void)M; (void)H; (void)G;
    return io == STRD_BF16 && (n == 64 || n == 128) && N >= 1;
}

int score_mamba_mfma(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, int n,
                     hipStream_t st) {
    // wide token tiles once there are enough of them to fill 256 CUs; narrow ones otherwise
    const bool wide = N >= 256 * 256;
    if (n == 128) return wide ? launch<128, 2>(B, C, dt, s, M, N, H, G, st) : launch<128, 1>(B, C, dt, s, M, N, H, G, st);
    if (n == 64) return wide ? launch<64, 2>(B, C, dt, s, M, N, H, G, st) : launch<64, 1>(B, C, dt, s, M, N, H, G, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
