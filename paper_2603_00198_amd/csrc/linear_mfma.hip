// strd_linear_mfma: out[T, Nd] = x[T, Kd] . w[Kd, Nd] (+ residual) on bf16 matrix cores with fp32
// accumulation -- the projections of a block (in-projection, out-projection onto the residual
// stream) as a kernel of this library: no handle, no allocation, nothing kept between calls.
//
// One workgroup owns a 256-token x 256-column tile of the output.  Eight computing waves, two per
// SIMD, as 2 token halves x 4 column quarters: a wave keeps a 128-token x 64-column block in 128
// accumulator registers (32 tiles of v_mfma_f32_16x16x32_bf16).  The product is computed transposed,
//     D[n, t] = sum_k w[k, n] x[t, k]       A = w, read from LDS with the transposing load (w is stored
//                                               with n contiguous, the operand needs k contiguous),
//                                           B = x rows, 16 bytes per lane,
// so a lane ends up with four consecutive columns of one token and stores 8 bytes at a time.
// Four copy waves, one per SIMD, do nothing but request the asynchronous global -> LDS copies (no
// register staging): w in stages of 32 rows of k, a ring of four, three stages ahead; x in blocks
// of 64 k (whole 128-byte lines of every token row), two blocks, one ahead.  A stage is one
// contraction step of the matrix instruction; one LDS-only barrier per stage.
//
// What bounds it: a CU takes in 64 KB per 64 of k (1/128 byte per flop at this tile size) through
// its path from L2, which delivers about 25 bytes per clock and CU however the copies are requested:
// 2600 clocks, against 2048 clocks of a SIMD's matrix pipe for the products.  The 16 x 16 x 32 form of
// the instruction matters: with 32 x 32 x 16 products (half as many operand reads) the same kernel
// needs 9.3 M clocks instead of 6.7 M -- long products and the copies do not overlap.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBT = 256;   // tokens per workgroup tile
constexpr int kBN = 256;   // output columns per workgroup tile
constexpr int kBK = 32;    // contraction depth per w stage (one step of the matrix instruction)
constexpr int kXK = 64;    // contraction depth per x block (two stages)
constexpr int kRingW = 4;  // w stages in LDS
constexpr int kRingX = 2;  // x blocks in LDS
constexpr int kNW = 8;     // computing waves
constexpr int kNCW = 4;    // copy waves
constexpr int kBand = 8;   // token tiles per band of the tile order

// x block [256 tokens][8 vectors + 2 pad]: pitch 40 words -- the 16-byte reads of 16 rows x 4 pieces run at
// 180 B/clk/CU (117 with one pad vector).  w stage [32 k][32 vectors + 4 pad]: pitch 144 words; the transposing
// reads run at 120 B/clk/CU at any pitch but 0 and 32 mod 64 words.  Both are filled 256 slots (4 copy waves)
// at a time: 10 rounds per x block; 4.5 rounds per w stage, which is given the room of 5 so that every copy
// wave issues the same number of copies per stage (the count of outstanding copies is what the waves wait on).
constexpr int kXV = 8, kXP = 10, kWV = 32, kWP = 36;
constexpr int kNX = 10, kNWc = 5;  // copies per copy wave: x block, w stage
constexpr int kXBytes = kBT * kXP * 16, kWBytes = kNWc * kNCW * 64 * 16;
constexpr int kWBase = kRingX * kXBytes;
constexpr int kLdsBytes = kWBase + kRingW * kWBytes;
static_assert(kBT * kXP == kNX * kNCW * 64 && kBK * kWP <= kNWc * kNCW * 64, "whole rounds of 256 slots");
static_assert(kLdsBytes <= 160 * 1024, "one workgroup must fit the 160 KB of LDS of a CU");

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// LDS reads by address, requested now and usable after the matching settle on the same registers (same
// contract as lds_issue_tr8 / lds_settle8: the kernel must not spill).
// w: the two transposing reads (rows + 0..3 and + 4..7) of four column tiles of 16, 32 bytes apart.
template <int ROW4>
__device__ __forceinline__ void issue_w(uint32_t a, strd_s16x4 (&r)[8]) {
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8 offset:%9\n\t"
        "ds_read_b64_tr_b16 %1, %8 offset:%10\n\t"
        "ds_read_b64_tr_b16 %2, %8 offset:%11\n\t"
        "ds_read_b64_tr_b16 %3, %8 offset:%12\n\t"
        "ds_read_b64_tr_b16 %4, %8 offset:%13\n\t"
        "ds_read_b64_tr_b16 %5, %8 offset:%14\n\t"
        "ds_read_b64_tr_b16 %6, %8 offset:%15\n\t"
        "ds_read_b64_tr_b16 %7, %8 offset:%16"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
        : "v"(a), "i"(0), "i"(ROW4), "i"(32), "i"(32 + ROW4), "i"(64), "i"(64 + ROW4), "i"(96), "i"(96 + ROW4)
        : "memory");
}
// x: four token tiles of 16, TILE bytes apart, starting at byte offset OFF
template <int OFF, int TILE>
__device__ __forceinline__ void issue_x(uint32_t a, bf16x8 (&r)[4]) {
    asm volatile(
        "ds_read_b128 %0, %4 offset:%5\n\t"
        "ds_read_b128 %1, %4 offset:%6\n\t"
        "ds_read_b128 %2, %4 offset:%7\n\t"
        "ds_read_b128 %3, %4 offset:%8"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(a), "i"(OFF), "i"(OFF + TILE), "i"(OFF + 2 * TILE), "i"(OFF + 3 * TILE)
        : "memory");
}
__device__ __forceinline__ void settle_wx(strd_s16x4 (&w)[8], bf16x8 (&x)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]), "+v"(x[0]),
                   "+v"(x[1]), "+v"(x[2]), "+v"(x[3])
                 :
                 : "memory");
}
__device__ __forceinline__ void settle_x(bf16x8 (&x)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]) : : "memory");
}
// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding (n < 64)
constexpr int vm_wait_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

__global__ __launch_bounds__((kNW + kNCW) * kWave) __attribute__((amdgpu_waves_per_eu(3, 3))) void linear_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, const bf16_t *residual, bf16_t *out, int T, int Kd, int Nd,
    int tiles_t, int tiles_n, int ntiles) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
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
    const int nk = Kd / kBK;  // even, at least 2

    if (wv >= kNW) {
        // ---- copy wave.  w stage s = w[32 s .., n0 ..]; x block j = x[t0 .., 64 j ..].  Rows past T and columns
        // past Nd re-read the last valid ones (their products are never stored). ----
        const int cw = wv - kNW;
        uint32_t xo[kNX], wo[kNWc];
        bool xok[kNX], wok[kNWc];
#pragma unroll
        for (int i = 0; i < kNX; ++i) {
            const int s = (i * kNCW + cw) * 64 + lane;
            const int xr = s / kXP, xc = s % kXP;
            xok[i] = xc < kXV;  // a lane on a pad slot copies nothing
            xo[i] = (uint32_t)min(t0 + xr, T - 1) * ((uint32_t)Kd * 2) + (uint32_t)min(xc, kXV - 1) * 16;
        }
#pragma unroll
        for (int i = 0; i < kNWc; ++i) {
            const int s = (i * kNCW + cw) * 64 + lane;
            const int wr = min(s / kWP, kBK - 1), wc = s % kWP;
            wok[i] = wc < kWV;  // slots past the stage re-copy its last row into the spare room
            wo[i] = (uint32_t)wr * ((uint32_t)Nd * 2) + (uint32_t)min(n0 / 8 + min(wc, kWV - 1), Nd / 8 - 1) * 16;
        }
        const char *xsrc = reinterpret_cast<const char *>(x);
        const char *wsrc = reinterpret_cast<const char *>(w);
        const size_t wstep = (size_t)kBK * Nd * 2;
        auto copy_x = [&](int slot) __attribute__((always_inline)) {  // the next x block in sequence
            unsigned char *xs = smem + slot * kXBytes;
#pragma unroll
            for (int i = 0; i < kNX; ++i)
                if (xok[i])
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(xsrc + xo[i]),
                                                     (__attribute__((address_space(3))) void *)(xs + (i * kNCW + cw) * 1024), 16, 0, 0);
            xsrc += kXK * 2;
        };
        auto copy_w = [&](int slot) __attribute__((always_inline)) {  // the next w stage in sequence
            unsigned char *ws = smem + kWBase + slot * kWBytes;
#pragma unroll
            for (int i = 0; i < kNWc; ++i)
                if (wok[i])
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wsrc + wo[i]),
                                                     (__attribute__((address_space(3))) void *)(ws + (i * kNCW + cw) * 1024), 16, 0, 0);
            wsrc += wstep;
        };
        // Copies land in the order they were requested, so "at most n outstanding" means everything but the
        // last n has landed.
        copy_x(0);
        copy_w(0);
        copy_w(1);
        if (nk > 2) {
            copy_w(2);
            __builtin_amdgcn_s_waitcnt(vm_wait_imm(2 * kNWc));  // x block 0 and w stage 0 have landed
        } else {
            __builtin_amdgcn_s_waitcnt(vm_wait_imm(kNWc));
        }
        lds_barrier();
        for (int kb = 0; kb < nk; ++kb) {
            // The barrier that ended stage kb - 1 freed its w slot and, for even kb, the x block before this one.
            if (kb + 3 < nk) {
                if ((kb & 1) == 0) {
                    copy_x(((kb >> 1) + 1) & (kRingX - 1));
                    copy_w((kb + 3) & (kRingW - 1));
                    // w stage kb + 1 has landed; w stages kb + 2, kb + 3 and the new x block may still travel
                    __builtin_amdgcn_s_waitcnt(vm_wait_imm(2 * kNWc + kNX));
                } else {
                    copy_w((kb + 3) & (kRingW - 1));
                    // x block (kb + 1) / 2, requested one stage ago, and w stage kb + 1 have landed
                    __builtin_amdgcn_s_waitcnt(vm_wait_imm(2 * kNWc));
                }
            } else {
                __builtin_amdgcn_s_waitcnt(vm_wait_imm(0));  // the last three stages: everything requested exists and lands
            }
            lds_barrier();
        }
        return;
    }

    // ---- computing wave: columns n0 + 64 wn .. + 63 of tokens t0 + 128 wt .. + 127.  x: lane (lr, lb) reads the 8
    // consecutive k at 8 lb of token row lr of a tile.  w: lane group lb passes rows 8 lb + lr / 4 (then + 4) and
    // columns 4 (lr % 4) of a 16-column tile and receives the k slots 8 lb .. 8 lb + 7 of column lr. ----
    const int wt = wv >> 2, wn = wv & 3;
    const int lr = lane & 15, lb = lane >> 4;
    constexpr int XPB = kXP * 16, WPB = kWP * 16;  // row pitches in bytes
    const uint32_t lds0 = lds_offset(smem);
    const uint32_t x_lane = lds0 + (uint32_t)((128 * wt + lr) * XPB + 16 * lb);
    const uint32_t w_lane = lds0 + (uint32_t)(kWBase + (8 * lb + (lr >> 2)) * WPB + (64 * wn + 4 * (lr & 3)) * 2);
    f32x4 acc[4][8];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int tb = 0; tb < 8; ++tb) acc[nt][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    lds_barrier();  // x block 0 and w stage 0 have landed
    for (int kb = 0; kb < nk; ++kb) {
        const uint32_t wa = w_lane + (uint32_t)(kb & (kRingW - 1)) * kWBytes;
        const uint32_t xa = x_lane + (uint32_t)((kb >> 1) & (kRingX - 1)) * kXBytes + (uint32_t)(kb & 1) * (kBK * 2);
        // the register budget of three waves per SIMD has room for the w fragments and half of the x fragments
        // of a stage: the second half is requested when the products of the first have been issued
        strd_s16x4 wr[8];
        bf16x8 xf[4];
        issue_w<4 * WPB>(wa, wr);
        issue_x<0, 16 * XPB>(xa, xf);
        settle_wx(wr, xf);
        bf16x8 af[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) af[nt] = tr_pair(wr[2 * nt], wr[2 * nt + 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[nt][tb] = mfma16(af[nt], xf[tb], acc[nt][tb]);
        __builtin_amdgcn_sched_barrier(0);
        issue_x<64 * XPB, 16 * XPB>(xa, xf);
        settle_x(xf);
        lds_barrier();  // every read of this stage has returned: its slots may be overwritten; the next stage has landed
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[nt][4 + tb] = mfma16(af[nt], xf[tb], acc[nt][4 + tb]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- outputs: acc[nt][tb][r] is column n0 + 64 wn + 16 nt + 4 lb + r of token t0 + 128 wt + 16 tb + lr ----
    const int nl = n0 + 64 * wn + 4 * lb;
#pragma unroll
    for (int tb = 0; tb < 8; ++tb) {
        const int t = t0 + 128 * wt + 16 * tb + lr;
        if (t >= T) continue;
        const size_t o = (size_t)t * Nd + nl;
        bf16_t *op = out + o;
        const bf16_t *rp = residual ? residual + o : nullptr;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            if (nl + 16 * nt >= Nd) continue;  // Nd is a multiple of 8: four columns are in or out together
            bf16x4 v;
            if (rp) {  // may be `out` itself: a lane reads what it then overwrites
                const bf16x4 r = *reinterpret_cast<const bf16x4 *>(rp + 16 * nt);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16_t)(acc[nt][tb][e] + (float)r[e]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (bf16_t)acc[nt][tb][e];
            }
            *reinterpret_cast<bf16x4 *>(op + 16 * nt) = v;
        }
    }
}

}  // namespace

bool linear_mfma_supported(int T, int Kd, int Nd, strd_dtype io) {
    // copies use 32-bit byte offsets into x and w
    return io == STRD_BF16 && T >= 1 && Kd >= kXK && Kd % kXK == 0 && Nd >= 8 && Nd % 8 == 0 &&
           (unsigned long long)T * Kd * 2 < (1ull << 32) && (unsigned long long)Kd * Nd * 2 < (1ull << 32) &&
           (long long)ceil_div(T, kBT) * ceil_div(Nd, kBN) < (1LL << 30);
}

int linear_mfma(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, hipStream_t st) {
    const size_t smem = (size_t)kLdsBytes;
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&linear_mfma_kernel), smem)) return STRD_EHIP;
    const int tiles_t = ceil_div(T, kBT), tiles_n = ceil_div(Nd, kBN), ntiles = tiles_t * tiles_n;
    linear_mfma_kernel<<<xcd_grid(ntiles), (kNW + kNCW) * kWave, smem, st>>>((const bf16_t *)x, (const bf16_t *)w,
                                                                            (const bf16_t *)residual, (bf16_t *)out, T, Kd, Nd,
                                                                            tiles_t, tiles_n, ntiles);
    return launch_status();
}

}  // namespace strd
