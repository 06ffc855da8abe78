// strd_linear_mfma: out[T, Nd] = x[T, Kd] . w[Kd, Nd] (+ residual) on bf16 matrix cores with fp32
// accumulation -- the projections of a block (in-projection, out-projection onto the residual
// stream) as a kernel of this library: no handle, no allocation, nothing kept between calls.
//
// One workgroup owns a 256-token x 256-column tile of the output and walks the contraction in
// stages of 64.  Eight waves, two per SIMD, as 2 token halves x 4 column quarters: a wave keeps a
// 128-token x 64-column block in 128 accumulator registers (v_mfma_f32_32x32x16_bf16, eight
// 32 x 32 tiles).  The product is computed transposed,
//     D[n, t] = sum_k w[k, n] x[t, k]       A = w, read from LDS with the transposing load (w is stored
//                                               with n contiguous, the operand needs k contiguous),
//                                           B = x rows, 16 bytes per lane,
// so a lane ends up with four consecutive columns of one token and stores 8 bytes at a time.
// Both operand tiles of a stage go global -> LDS asynchronously (no register staging), double
// buffered: the copies of stage s + 1 are requested when stage s starts and waited for when it
// ends, one LDS-only barrier per stage.  The LDS reads of a 16-deep step are requested one step
// ahead of its eight products; the last step's products run after the barrier, under the first
// reads of the next stage.
//
// What bounds it: a CU takes in 64 KB per stage (1/128 byte per flop at this tile size) through its
// path from L2, which delivers about 25 bytes per clock and CU however the copies are requested; the
// products of a stage need 2048 clocks of a SIMD's matrix pipe, the copies 2600 clocks of that path.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBT = 256;  // tokens per workgroup tile
constexpr int kBN = 256;  // output columns per workgroup tile
constexpr int kBK = 64;   // contraction depth per stage
constexpr int kNW = 8;    // waves: 2 token halves x 4 column quarters
constexpr int kBand = 8;  // token tiles per band of the tile order

struct GemmLds {
    // x stage [token][k]: rows of 8 vectors + 1 pad, pitch 36 words: 16-byte reads of 16 rows touch all 64 banks.
    // w stage [k][n]: rows of 32 vectors + 4 pad, pitch 144 words = 16 mod 64: the four rows that a half wave
    // passes to a transposing read lie 16 banks apart.  (No bank conflicts by counter.)
    using XT = AsyncTile<kBT, kBK / 8, kNW, 1, true>;
    using WT = AsyncTile<kBK, kBN / 8, kNW, 4, true>;
    struct alignas(16) Stage {
        bf16_t x[XT::kBytes / 2];
        bf16_t w[WT::kBytes / 2];
    };
    Stage st[2];
};
static_assert(sizeof(GemmLds) <= 160 * 1024, "one workgroup must fit the 160 KB of LDS of a CU");

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The fragments of one 16-deep step: 4 transposing reads (w, two column tiles of 32) and 4 16-byte
// reads (x, four token tiles of 32), requested together; usable after settle_frags on the same
// registers (same contract as lds_issue_tr8 / lds_settle8: the kernel must not spill).
struct Frags {
    strd_s16x4 w[4];
    bf16x8 x[4];
};
template <int WOFF, int XOFF, int WROW4, int XTILE>
__device__ __forceinline__ void issue_frags(uint32_t wa, uint32_t xa, Frags &f) {
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8 offset:%10\n\t"
        "ds_read_b64_tr_b16 %1, %8 offset:%11\n\t"
        "ds_read_b64_tr_b16 %2, %8 offset:%12\n\t"
        "ds_read_b64_tr_b16 %3, %8 offset:%13\n\t"
        "ds_read_b128 %4, %9 offset:%14\n\t"
        "ds_read_b128 %5, %9 offset:%15\n\t"
        "ds_read_b128 %6, %9 offset:%16\n\t"
        "ds_read_b128 %7, %9 offset:%17"
        : "=&v"(f.w[0]), "=&v"(f.w[1]), "=&v"(f.w[2]), "=&v"(f.w[3]), "=&v"(f.x[0]), "=&v"(f.x[1]), "=&v"(f.x[2]), "=&v"(f.x[3])
        : "v"(wa), "v"(xa), "i"(WOFF), "i"(WOFF + WROW4), "i"(WOFF + 64), "i"(WOFF + 64 + WROW4), "i"(XOFF), "i"(XOFF + XTILE),
          "i"(XOFF + 2 * XTILE), "i"(XOFF + 3 * XTILE)
        : "memory");
}
__device__ __forceinline__ void settle_frags(Frags &f) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.w[0]), "+v"(f.w[1]), "+v"(f.w[2]), "+v"(f.w[3]), "+v"(f.x[0]), "+v"(f.x[1]), "+v"(f.x[2]), "+v"(f.x[3])
                 :
                 : "memory");
}

__global__ __launch_bounds__(kNW * kWave) __attribute__((amdgpu_waves_per_eu(2, 2))) void linear_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, const bf16_t *residual, bf16_t *out, int T, int Kd, int Nd,
    int tiles_t, int tiles_n, int ntiles) {
    using XT = GemmLds::XT;
    using WT = GemmLds::WT;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    GemmLds &lds = *reinterpret_cast<GemmLds *>(smem_raw);
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // Tile order: consecutive units run on one XCD (one L2); they walk down a band of kBand token tiles and
    // then move one column tile on, so the 32 workgroups an XCD runs at a time share 8 x tiles and 4 w tiles
    // (4/5 of their requests hit in that L2).
    const int unit = xcd_swizzle(blockIdx.x, ntiles);
    if (unit >= ntiles) return;
    const int band_units = kBand * tiles_n;
    const int band = unit / band_units, within = unit - band * band_units;
    const int rows = min(kBand, tiles_t - kBand * band);
    const int tn = within / rows, tt = kBand * band + within % rows;
    const int t0 = tt * kBT, n0 = tn * kBN;
    const int nk = Kd / kBK;

    // ---- copies: a stage is x[t0 .., 64 kb ..] and w[64 kb .., n0 ..]; rows past T and columns past Nd
    // re-read the last valid ones (their products are never stored) ----
    uint32_t xo[XT::kIssues], wo[WT::kIssues];
#pragma unroll
    for (int i = 0; i < XT::kIssues; ++i) {
        int row, cv;
        XT::slot(wv, lane, i, row, cv);
        xo[i] = (uint32_t)min(t0 + row, T - 1) * ((uint32_t)Kd * 2) + (uint32_t)cv * 16;
    }
#pragma unroll
    for (int i = 0; i < WT::kIssues; ++i) {
        int row, cv;
        WT::slot(wv, lane, i, row, cv);
        wo[i] = (uint32_t)row * ((uint32_t)Nd * 2) + (uint32_t)min(n0 / 8 + cv, Nd / 8 - 1) * 16;
    }
    const char *xsrc = reinterpret_cast<const char *>(x);
    const char *wsrc = reinterpret_cast<const char *>(w);
    const size_t wstep = (size_t)kBK * Nd * 2;
    auto stage = [&](int s) __attribute__((always_inline)) {  // requests the next stage in sequence
#pragma unroll
        for (int i = 0; i < XT::kIssues; ++i) XT::issue(xsrc + xo[i], lds.st[s].x, wv, i);
#pragma unroll
        for (int i = 0; i < WT::kIssues; ++i) WT::issue(wsrc + wo[i], lds.st[s].w, wv, i);
        xsrc += kBK * 2;
        wsrc += wstep;
    };

    // ---- this wave's block: columns n0 + 64 wn .. + 63 of tokens t0 + 128 wt .. + 127 ----
    const int wt = wv >> 2, wn = wv & 3;
    const int tl = lane & 31, half = lane >> 5, vb = lane >> 4, vr = lane & 15;
    constexpr int XPB = XT::kPitch * 2, WPB = WT::kPitch * 2;  // row pitches in bytes
    // x: row = token, 8 consecutive k at 16 ks + 8 half.  w: a group of 16 lanes passes rows k0 + vr / 4 and
    // columns c0 + 4 (vr % 4) and receives [k0 .. k0 + 3][c0 + vr]; lane groups 0, 1 take the two column
    // halves of a 32-column tile, the lane halves the k slots 0-7 and 8-15 (rows + 0..3 and + 4..7: two reads).
    const uint32_t x_lane = (uint32_t)((128 * wt + tl) * XPB + 16 * half);
    const uint32_t w_lane = (uint32_t)((8 * (vb >> 1) + (vr >> 2)) * WPB + (64 * wn + 16 * (vb & 1) + 4 * (vr & 3)) * 2);
    f32x16 acc[2][4];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nt][tb][i] = 0.f;
    auto products = [&](Frags &f) __attribute__((always_inline)) {
        const bf16x8 a0 = tr_pair(f.w[0], f.w[1]), a1 = tr_pair(f.w[2], f.w[3]);
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            acc[0][tb] = mfma32(a0, f.x[tb], acc[0][tb]);
            acc[1][tb] = mfma32(a1, f.x[tb], acc[1][tb]);
        }
    };

    stage(0);
    async_tile_wait();
    lds_barrier();
    Frags fa, fb;
    issue_frags<0, 0, 4 * WPB, 32 * XPB>(lds_offset(lds.st[0].w) + w_lane, lds_offset(lds.st[0].x) + x_lane, fa);
    for (int kb = 0; kb < nk; ++kb) {
        const int cur = kb & 1;
        const bool more = kb + 1 < nk;  // uniform
        if (more) stage(cur ^ 1);       // the buffer every wave left at the last barrier
        const uint32_t wa = lds_offset(lds.st[cur].w) + w_lane, xa = lds_offset(lds.st[cur].x) + x_lane;
        // the scheduling barriers keep each request ahead of the products it travels under
        settle_frags(fa);
        issue_frags<16 * WPB, 32, 4 * WPB, 32 * XPB>(wa, xa, fb);
        __builtin_amdgcn_sched_barrier(0);
        products(fa);
        __builtin_amdgcn_sched_barrier(0);
        settle_frags(fb);
        issue_frags<32 * WPB, 64, 4 * WPB, 32 * XPB>(wa, xa, fa);
        __builtin_amdgcn_sched_barrier(0);
        products(fb);
        __builtin_amdgcn_sched_barrier(0);
        settle_frags(fa);
        issue_frags<48 * WPB, 96, 4 * WPB, 32 * XPB>(wa, xa, fb);
        __builtin_amdgcn_sched_barrier(0);
        products(fa);
        __builtin_amdgcn_sched_barrier(0);
        settle_frags(fb);   // every read of this stage has returned
        async_tile_wait();  // this wave's share of the next stage has landed
        lds_barrier();      // ... and everybody's; this stage may be overwritten
        if (more) issue_frags<0, 0, 4 * WPB, 32 * XPB>(lds_offset(lds.st[cur ^ 1].w) + w_lane, lds_offset(lds.st[cur ^ 1].x) + x_lane, fa);
        __builtin_amdgcn_sched_barrier(0);
        products(fb);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- outputs: acc[nt][tb][4 b + r] is column n0 + 64 wn + 32 nt + 8 b + 4 half + r of token
    // t0 + 128 wt + 32 tb + tl (accumulator layout of the 32 x 32 product) ----
    const int nl = n0 + 64 * wn + 4 * half;
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int t = t0 + 128 * wt + 32 * tb + tl;
        if (t >= T) continue;
        const size_t o = (size_t)t * Nd + nl;
        bf16_t *op = out + o;
        const bf16_t *rp = residual ? residual + o : nullptr;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (nl + 32 * nt + 8 * b >= Nd) continue;  // Nd is a multiple of 8: four columns are in or out together
                bf16x4 v;
                if (rp) {  // may be `out` itself: a lane reads what it then overwrites
                    const bf16x4 r = *reinterpret_cast<const bf16x4 *>(rp + 32 * nt + 8 * b);
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(acc[nt][tb][4 * b + e] + (float)r[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (bf16_t)acc[nt][tb][4 * b + e];
                }
                *reinterpret_cast<bf16x4 *>(op + 32 * nt + 8 * b) = v;
            }
    }
}

}  // namespace

bool linear_mfma_supported(int T, int Kd, int Nd, strd_dtype io) {
    // copies use 32-bit byte offsets into x and w
    return io == STRD_BF16 && T >= 1 && Kd >= kBK && Kd % kBK == 0 && Nd >= 8 && Nd % 8 == 0 &&
           (unsigned long long)T * Kd * 2 < (1ull << 32) && (unsigned long long)Kd * Nd * 2 < (1ull << 32) &&
           (long long)ceil_div(T, kBT) * ceil_div(Nd, kBN) < (1LL << 30);
}

int linear_mfma(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, hipStream_t st) {
    const size_t smem = sizeof(GemmLds);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&linear_mfma_kernel), smem)) return STRD_EHIP;
    const int tiles_t = ceil_div(T, kBT), tiles_n = ceil_div(Nd, kBN), ntiles = tiles_t * tiles_n;
    linear_mfma_kernel<<<xcd_grid(ntiles), kNW * kWave, smem, st>>>((const bf16_t *)x, (const bf16_t *)w, (const bf16_t *)residual,
                                                                   (bf16_t *)out, T, Kd, Nd, tiles_t, tiles_n, ntiles);
    return launch_status();
}

}  // namespace strd
