// attn_prefill on bf16 matrix cores: causal softmax attention with grouped-query heads (paper
// App. "Attention via Kernel Functions", first equation), flash-style: the score matrix is
// produced and consumed tile by tile with a running max and sum per query.
//
// One workgroup = NW waves = one query head x 32 * NW consecutive query positions; wave w owns 32
// of them as two tiles of 16.  Tiles are computed transposed (v_mfma_f32_16x16x32_bf16):
//     S^T[key, t] = K_tile . Q^T        A = key rows from LDS, B = query fragments in registers
//     O^T[d,  t] += V_tile^T . P^T      A = V read with the transposing LDS load, B = P^T
// so a lane owns one query column of each tile: its running max, running sum and the rescale
// factor are per-lane scalars (shared by the four lane groups that hold different keys of the
// query), and the fp32 score accumulators of two 16-key tiles, converted to bf16, are already
// laid out as the B operand of the second product: lane group lb holds keys 4 lb .. 4 lb + 3 of
// both tiles, i.e. the 8 contraction slots of a 32-key step in the order (4 lb + s, 16 + 4 lb + s),
// and V is read with the matching key permutation.
// The 16 x 16 x 32 form of the product is deliberate: with 32 x 32 x 16 products (half as many
// operand reads) the asynchronous K / V copies and the matrix pipe do not overlap -- the same
// kernel took 18 % longer at 33 K tokens.
// K and V stream through LDS in chunks of KC keys, double-buffered, shared by the waves; the next
// chunk is copied global -> LDS asynchronously (no register staging) during the current one.
// Two shapes: 4 waves that request their own copies and 64-key chunks (two workgroups per CU) for
// short sequences; 8 computing waves, 4 copy waves and 128-key chunks (one workgroup per CU) for
// long ones.  Workgroups are issued longest-first (last query block first), the query heads of one
// kv group back to back on one XCD.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.f;  // log2 of how far a probability may exceed 1 before the reference moves

// K rows are read 16 bytes per lane, lane = (row lane % 16, piece lane / 16), V with the transposing load,
// 8 consecutive rows per half wave: both run fastest at a row pitch of 8 words modulo 32 (two pad
// vectors, never copied): 180 and 118 bytes per clock and CU, against 117 and 108 with one pad vector.
// NC = number of waves that fill the tiles.
template <int D, int NC, int KC>
struct Tile {
    using A = AsyncTile<KC, D / 8, NC, 2, true>;
    static constexpr int kPitch = A::kPitch;
    struct alignas(16) Half {
        bf16_t e[A::kBytes / 2];
        __device__ __forceinline__ const bf16_t *at(int r, int c) const { return e + r * kPitch + c; }
    };
    Half k[2];
    Half v[2];
};

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// NW computing waves and NC copy waves; NC = 0: the computing waves request the copies themselves.
template <int D, int NW, int NC, int KC>
__global__ __launch_bounds__((NW + NC) * kWave) __attribute__((amdgpu_waves_per_eu(2, NC ? 3 : 2))) void attn_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v, bf16_t *__restrict__ o, int T,
    int Hq, int Hkv, float scale2, int nqb, int xcd_map) {
    constexpr int KS = D / 32, DT = D / 16, kBM = 32 * NW;
    using TileT = Tile<D, NC ? NC : NW, KC>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    TileT &lds = *reinterpret_cast<TileT *>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, lr = lane & 15, lb = lane >> 4;
    const float lazy_raw = kLazy / scale2;  // the slack of the softmax reference, in raw score units
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, in a scalar register
    // Workgroup b runs on XCD b % 8, each with an L2 of its own.  When the kv heads divide evenly over
    // the XCDs, all query heads and query blocks of one kv head go to one XCD, so its K and V stream
    // through one L2 (and the query heads of the group, issued back to back, share each chunk there)
    // instead of through all eight; otherwise heads are simply dealt round.  Longest blocks first.
    // xcd_map: 0, or 1 + log2(kv heads per XCD) + 8 * log2(query heads per kv head) -- shifts and
    // masks only, so the indices stay in scalar registers.
    int h, qb, kvh;
    if (xcd_map) {
        const int ps = (xcd_map - 1) & 7, gs = (xcd_map - 1) >> 3;
        const int xcd = blockIdx.x % kXcd, j = blockIdx.x / kXcd, r = j >> ps;
        kvh = xcd + kXcd * (j & ((1 << ps) - 1));
        h = (kvh << gs) + (r & ((1 << gs) - 1));
        qb = nqb - 1 - (r >> gs);
    } else {
        h = blockIdx.x % Hq;
        qb = nqb - 1 - blockIdx.x / Hq;
        kvh = h / (Hq / Hkv);
    }
    const int t0 = qb * kBM;
    const int tq0 = t0 + 32 * w + lr, tq1 = tq0 + 16;  // this lane's query positions (tiles 0 and 1)
    // first query of the wave, in a scalar register so that tests on it are real branches (the wave
    // index comes from threadIdx, which the compiler cannot prove uniform)
    const int wq0 = __builtin_amdgcn_readfirstlane(t0 + 32 * w);
    const int wmax = min(T - 1, wq0 + 31);       // last key any query of the wave may see
    const int nkeys = min(T, t0 + kBM);
    const int nchunk = (nkeys + KC - 1) / KC;

    // K / V chunks go global -> LDS directly, one chunk ahead of the products.  Requesting a copy
    // blocks a wave for as long as the CU's copy path is busy with earlier ones (about half of the
    // time at long sequences), so there the requests are kept out of the waves that feed the matrix
    // cores: the last NC waves of the workgroup do nothing else.  With NC = 0 every computing wave
    // requests its share.  The slots of a lane are recomputed for every chunk (a few integer
    // operations) rather than held in registers.
    using AT = typename TileT::A;
    const int cw = NC ? w - NW : w;
    const uint32_t kv_row = (uint32_t)Hkv * D * 2;
    const uint32_t kv_col = (uint32_t)kvh * D * 2;
    int next_chunk = 0;
    auto stage = [&](int b) __attribute__((always_inline)) {  // requests the next chunk in sequence; rows past T re-read row T - 1
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            int row, cv;
            AT::slot(cw, lane, i, row, cv);
            const uint32_t off = (uint32_t)min(next_chunk * KC + row, T - 1) * kv_row + kv_col + (uint32_t)cv * 16;
            AT::issue(reinterpret_cast<const char *>(k) + off, &lds.k[b], cw, i);
        }
#pragma unroll
        for (int i = 0; i < AT::kIssues; ++i) {
            int row, cv;
            AT::slot(cw, lane, i, row, cv);
            const uint32_t off = (uint32_t)min(next_chunk * KC + row, T - 1) * kv_row + kv_col + (uint32_t)cv * 16;
            AT::issue(reinterpret_cast<const char *>(v) + off, &lds.v[b], cw, i);
        }
        ++next_chunk;
    };
    if (NC > 0 && w >= NW) {  // copy wave
        stage(0);
        async_tile_wait();
        lds_barrier();
        for (int chunk = 0; chunk < nchunk; ++chunk) {
            stage((chunk & 1) ^ 1);  // chunk + 1 (past the last chunk: clamped rows, never read)
            async_tile_wait();
            lds_barrier();
        }
        return;
    }

    // query fragments: B operand, column = query lr of the tile, k slots d = 32 ks + 8 lb ..
    bf16x8 bq[2][KS];
    {
        const bf16_t *qp0 = q + ((size_t)min(tq0, T - 1) * Hq + h) * D + 8 * lb;
        const bf16_t *qp1 = q + ((size_t)min(tq1, T - 1) * Hq + h) * D + 8 * lb;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bq[0][ks] = *reinterpret_cast<const bf16x8 *>(qp0 + 32 * ks);
            bq[1][ks] = *reinterpret_cast<const bf16x8 *>(qp1 + 32 * ks);
        }
    }

    // O^T tiles: oacc[dt][qt][r] = channel 16 dt + 4 lb + r of query (qt, lr)
    f32x4 oacc[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt][0] = oacc[dt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    // per query tile; l_run: this lane group's share of the row sum
    float m_run[2] = {-INFINITY, -INFINITY}, m_neg[2] = {0.f, 0.f}, l_run[2] = {0.f, 0.f};

    constexpr int kRowB = TileT::kPitch * 2;  // row pitch of the tiles in bytes
    if (NC == 0) {
        stage(0);
        async_tile_wait();
    }
    lds_barrier();  // chunk 0 has landed
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int cur = chunk & 1;
        if (NC == 0) stage(cur ^ 1);  // chunk + 1 (past the last chunk: clamped rows, never read)
#pragma unroll
        for (int kt = 0; kt < KC / 32; ++kt) {
            const int kb = chunk * KC + 32 * kt;
            if (kb <= wmax) {  // uniform per wave
                // all key fragments of the 32 keys first (one LDS round trip, not one per product):
                // A operand, row = key lr of a 16-key tile, k slots d = 32 ks + 8 lb ..
                bf16x8 kf[2][KS];
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        kf[j][ks] = *reinterpret_cast<const bf16x8 *>(lds.k[cur].at(32 * kt + 16 * j + lr, 32 * ks + 8 * lb));
                __builtin_amdgcn_sched_barrier(0);
                // sacc[qt][j][r] = score of key kb + 16 j + 4 lb + r for query (qt, lr)
                f32x4 sacc[2][2];
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) sacc[qt][0] = sacc[qt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                // products first: the other wave of the SIMD is most likely in its softmax, and a
                // matrix instruction that waits behind its vector instructions leaves the matrix pipe idle
                __builtin_amdgcn_s_setprio(2);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int qt = 0; qt < 2; ++qt) sacc[qt][j] = mfma16(kf[j][ks], bq[qt][ks], sacc[qt][j]);
                __builtin_amdgcn_s_setprio(0);
                // the transposed V fragments are requested now and arrive during the softmax: lane group lb
                // passes rows 4 lb + lr / 4 (then + 16) and columns 4 (lr % 4) of a 16-channel tile and
                // receives, for channel lr, the keys 4 lb .. 4 lb + 3 (then 16 + 4 lb ..): the slot order of P
                // (64 channels now; the other 64 are requested after the softmax, when the score registers are free)
                strd_s16x4 vr8[DT / 4][8];
                const bf16_t *vp = lds.v[cur].at(32 * kt + 4 * lb + (lr >> 2), 4 * (lr & 3));
                lds_issue_tr8<0, 16 * kRowB, 32, 16 * kRowB + 32, 64, 16 * kRowB + 64, 96, 16 * kRowB + 96>(vp, vr8[0]);
                if (kb + 31 > wq0) {  // uniform: some (key, query) pair of the block is masked
                    asm volatile("" ::);  // keeps this a branch: folded into selects it would run for every block
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int key = kb + 16 * j + 4 * lb + r;
                            if (key > tq0) sacc[0][j][r] = -INFINITY;
                            if (key > tq1) sacc[1][j][r] = -INFINITY;
                        }
                }
                float tm[2];  // max of this lane's 8 raw scores per query tile
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    float t = sacc[qt][0][0];
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) t = fmaxf(t, sacc[qt][j][r]);
                    tm[qt] = t;
                }
                // m_run (raw units) is the reference the exponentials are taken against, common to the four
                // lane groups of a query.  Softmax does not care which reference is used, so it follows
                // the running max lazily: it moves (and the accumulators are rescaled, and the groups
                // talk) only when some lane sees a score more than 2^kLazy above it; until then the
                // probabilities are merely allowed to reach 2^kLazy instead of 1.
                if (__any(tm[0] > m_run[0] + lazy_raw || tm[1] > m_run[1] + lazy_raw)) {
#pragma unroll
                    for (int qt = 0; qt < 2; ++qt) {
                        float t = tm[qt];
                        t = fmaxf(t, __shfl_xor(t, 16, kWave));
                        t = fmaxf(t, __shfl_xor(t, 32, kWave));
                        const float nm = fmaxf(m_run[qt], t);  // finite: key 0 is visible to every query
                        const float corr = ex2((m_run[qt] - nm) * scale2);
                        l_run[qt] *= corr;
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) oacc[dt][qt] *= corr;
                        m_run[qt] = nm;
                        m_neg[qt] = -nm * scale2;
                    }
                }
                // The row sum is taken of the probabilities as they enter the second product, i.e. rounded to
                // bf16 (numerator and denominator then carry the same rounding), two at a time.
                bf16x8 pf[2];
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            pf[qt][4 * j + r] = (bf16_t)ex2(fmaf(sacc[qt][j][r], scale2, m_neg[qt]));  // 2^((s - m) * scale * log2 e)
                    float ps = l_run[qt];
#pragma unroll
                    for (int e = 0; e < 8; e += 2)
                        ps = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{pf[qt][e], pf[qt][e + 1]}, bf16x2{(bf16_t)1.f, (bf16_t)1.f}, ps, false);
                    l_run[qt] = ps;
                }
#pragma unroll
                for (int dp = 1; dp < DT / 4; ++dp)
                    lds_issue_tr8<0, 16 * kRowB, 32, 16 * kRowB + 32, 64, 16 * kRowB + 64, 96, 16 * kRowB + 96>(vp + 64 * dp, vr8[dp]);
                __builtin_amdgcn_s_setprio(2);
#pragma unroll
                for (int dp = 0; dp < DT / 4; ++dp) {
                    strd_s16x4(&r)[8] = vr8[dp];
                    if (dp + 1 < DT / 4)
                        lds_settle8_but<8 * (DT / 4 - 1)>(r);  // LDS reads return in order: the later batch may still travel
                    else
                        lds_settle8(r);
#pragma unroll
                    for (int dd = 0; dd < 4; ++dd) {
                        const bf16x8 vf = tr_pair(r[2 * dd], r[2 * dd + 1]);
                        oacc[4 * dp + dd][0] = mfma16(vf, pf[0], oacc[4 * dp + dd][0]);
                        oacc[4 * dp + dd][1] = mfma16(vf, pf[1], oacc[4 * dp + dd][1]);
                    }
                }
                __builtin_amdgcn_s_setprio(0);
            }
        }
        if (NC == 0) async_tile_wait();
        lds_barrier();  // chunk + 1 has landed, every wave is done with this one
    }

#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float l_tot = l_run[qt];
        l_tot += __shfl_xor(l_tot, 16, kWave);
        l_tot += __shfl_xor(l_tot, 32, kWave);
        const int tq = qt ? tq1 : tq0;
        if (tq < T) {
            const float inv = 1.f / l_tot;
            bf16_t *op = o + ((size_t)tq * Hq + h) * D + 4 * lb;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                bf16x4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (bf16_t)(oacc[dt][qt][e] * inv);
                *reinterpret_cast<bf16x4 *>(op + 16 * dt) = out;
            }
        }
    }
}

template <int D, int NW, int NC, int KC>
int launch(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, float scale, hipStream_t st) {
    const size_t smem = sizeof(Tile<D, NC ? NC : NW, KC>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&attn_mfma_kernel<D, NW, NC, KC>), smem))
        return STRD_EHIP;
    const int nqb = ceil_div(T, 32 * NW);
    // XCD-aware order when the kv heads per XCD and the query heads per kv head are powers of two
    const int per = Hkv / kXcd, gq = Hq / Hkv;
    const bool pow2 = Hkv % kXcd == 0 && (per & (per - 1)) == 0 && (gq & (gq - 1)) == 0 && per <= 128;
    const int xcd_map = pow2 ? 1 + __builtin_ctz(per) + 8 * __builtin_ctz(gq) : 0;
    attn_mfma_kernel<D, NW, NC, KC><<<nqb * Hq, (NW + NC) * kWave, smem, st>>>((const bf16_t *)q, (const bf16_t *)k,
                                                                        (const bf16_t *)v, (bf16_t *)o, T, Hq, Hkv,
                                                                        scale * kLog2e, nqb, xcd_map);
    return launch_status();
}

}  // namespace

bool attn_mfma_supported(int T, int Hq, int Hkv, int d, strd_dtype io) {
    // staging uses 32-bit byte offsets into K and V
    return io == STRD_BF16 && T >= 1 && (d == 64 || d == 128) && (long long)ceil_div(T, 128) * Hq < (1LL << 30) &&
           (unsigned long long)(T + 2 * 128) * Hkv * d * 2 < (1ull << 32);
}

int attn_mfma(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d, float scale,
              hipStream_t st) {
    // Long sequences: 8 computing waves (256 queries) per workgroup share 128-key chunks that 4 copy
    // waves bring in, one workgroup per CU -- half the K/V copies per query, a barrier every four
    // tiles instead of every two, and no computing wave ever blocks on the copy path (12 % faster
    // at 33 K tokens than the other form).  Short ones keep 4 waves that copy for themselves and
    // 64-key chunks, which makes twice as many workgroups; the crossover lies near 1.5 workgroups of
    // the long form per CU.
    const bool big = (long long)ceil_div(T, 256) * Hq >= 384;
    if (d == 128) return big ? launch<128, 8, 4, 128>(q, k, v, o, T, Hq, Hkv, scale, st) : launch<128, 4, 0, 64>(q, k, v, o, T, Hq, Hkv, scale, st);
    if (d == 64) return big ? launch<64, 8, 4, 128>(q, k, v, o, T, Hq, Hkv, scale, st) : launch<64, 4, 0, 64>(q, k, v, o, T, Hq, Hkv, scale, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
