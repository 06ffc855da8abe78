// ssd_prefill on bf16 matrix cores: the Mamba-2 recurrence (paper Eqs. "ssm_state_update",
// "ssm_output") in its chunked form, i.e. the unrolled sum (Eq. "ssm_unrolled") split at
// 64-token boundaries, with the recurrent state kept in registers for the whole sequence.
//
// Decomposition.  One workgroup (12 waves) owns one head h and a slab of 32 of its P channels
// and walks the sequence in 64-token steps; nothing but x, dt, B, C is read from HBM and
// nothing but y (and the final state) is written.  Per step, with l_t the in-step cumulative
// sum of dt*A (in log2 units) and all tiles staged in LDS:
//   (a) G^T[j,t] = b_j . c_t                        MFMA, contraction over the state dim n
//   (b) M^T[j,t] = G^T[j,t] * 2^(l_t-l_j) * dt_j  for j <= t, else 0     (fp32, then bf16)
//   (c) Y^T[p,t] = sum_j x_j[p] M^T[j,t]             MFMA, contraction over tokens
//   (d) Y^T[p,t] += 2^(l_t) * sum_n S[p,n] c_t[n]    MFMA, S = state before the step (bf16 copy)
//   (e) S^T[n,p] = 2^(l_Q) S^T[n,p] + sum_j b_j[n] (w_j x_j[p]),  w_j = dt_j 2^(l_Q-l_j)   MFMA
// Every MFMA is v_mfma_f32_16x16x32_bf16.  Results are kept "token on the lane" (columns of
// the accumulator tiles are tokens) so every token-dependent factor is one scalar per lane.
// Operands whose contraction index is the token (x in (c), b and w*x in (e)) are read from
// their token-major LDS tiles with the transposing LDS read (ds_read_b64_tr_b16).
//
// Roles.  Waves 0-3 ("output waves") compute (a)-(d), wave w for tokens 16w..16w+15 of the
// step; causality makes wave 3 do four times the (a)-(c) work of wave 0.  Waves 4-7 ("state
// waves") own the state rows for (e) in roughly the opposite proportion (2, 3, 2, 1 tiles of 16
// rows of n when n = 128), because wave 4+i shares a SIMD with wave i.
//
// Memory.  Every input reaches LDS by asynchronous global -> LDS copies, far enough ahead to cover
// HBM latency with only one workgroup per CU: three copy waves (9-11) request a third of the B and
// C tiles each, three steps ahead (ring of 3: a tile has landed two steps before its step, is read
// into registers during the step before its step and its slot is refilled during its own step; the
// tiles are shared by the 32 workgroups of a group through the XCD's L2); a helper wave (8)
// requests x three steps ahead (ring of 4) and dt four steps ahead (ring of 5), turns dt into the
// scan l_t, the key factors of (b) and the weights w_j two steps ahead and, in gather mode, keeps
// the row tables.  Issuing a copy costs a wave 50-100 ns, which is why the copies are spread over
// four waves that do nothing else.  Every computing wave fetches the operands that come from the
// tiles alone one step early: the output waves request the B / C / x fragments of the next step
// right after (d) and compute its (a) in the tail of the step; the state waves read their b^T and
// x fragments of the next step in the tail, weight the x fragments with w_j in registers and start
// the next step with the products of (e), so the new state copy is published early.  The bf16
// state copy is double-buffered.  One workgroup barrier per step.  Rows past T are copies of the
// last row with dt = 0, which makes them inert in (b)-(e); their y rows are not stored.  Each wave
// runs a straight-line specialisation (compile-time trip counts).
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kQ = 64;         // tokens per step
constexpr int kPB = 32;        // channels of the head per workgroup
constexpr int kCopyWaves = 3;
constexpr int kThreads = 64 * (9 + kCopyWaves);  // 4 output waves + 4 state waves + 1 helper wave + the copy waves
constexpr float kLog2e = 1.4426950408889634f;

constexpr int kXRing = 4;   // x tiles in LDS (requested kXRing - 1 steps ahead)
constexpr int kDtRing = 5;  // dt rows in LDS (requested kDtRing - 1 steps ahead)

template <int NS>
struct Lds {
    using BC = AsyncTile<kQ, NS / 8, kCopyWaves, 2, true>;  // B / C tile, filled by the copy waves, 2 pad vectors per row
    using XT = AsyncTile<kQ, kPB / 8, 1, 1, true>;  // x tile of the slab, filled by one wave, 1 pad vector per row
    static constexpr int kCP = BC::kPitch;    // bf16 elements per row of the B / C tiles
    static constexpr int kXP = XT::kPitch;    // bf16 elements per row of the x tiles
    static constexpr int kSP = NS + 8;        // bf16 elements per row of the state copy
    struct alignas(16) TileBC {
        bf16_t c[BC::kBytes / 2];
        bf16_t b[BC::kBytes / 2];
    };
    struct alignas(16) TileX {
        bf16_t x[XT::kBytes / 2];
    };
    struct alignas(16) Scan {
        float ell[kQ];  // inclusive cumulative sum of dt*A*log2(e) inside the step
        float dtv[kQ];  // dt (0 past the end of the sequence)
        float fw[96];   // key factors of query block W = 1..3 at fw_at(W): dt_j * 2^(l_{16W-1} - l_j), j < 16W
        float w[kQ];    // weights of the state update: w_j = dt_j * 2^(l_Q - l_j)
    };
    static constexpr int fw_at(int W) { return W <= 1 ? 0 : W == 2 ? 16 : 48; }
    TileBC bc[3];
    TileX xr[kXRing];
    float dt[kDtRing][kQ];
    uint32_t rowtab[4][kQ];  // gather mode: source row of every token of steps q, q % 4 = slot
    int32_t rawidx[4][kQ];   // gather mode: entries of the kept-index list for steps q, q % 4 = slot
    Scan scan[3];  // made two steps ahead
    bf16_t s[2][kPB][kSP];  // state before the step, [p][n]
};

static_assert(sizeof(Lds<128>) <= 160 * 1024, "one workgroup must fit the 160 KB of LDS of a CU");

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
// value of lane `l` (compile-time constant) in every lane, through a scalar register
__device__ __forceinline__ float read_lane_f32(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// The four token-contracted fragments of an x tile (pr = token half, pt = channel half).
// Token slots of a fragment: s < 4 is token 32*pr + 4*lb + s, s >= 4 adds 16.
// Issued early (issue_x_frags), usable after take_x_frags.
template <int PITCH>
__device__ __forceinline__ void issue_x_frags(const bf16_t *xt, int lr, int lb, strd_s16x4 (&r)[8]) {
    constexpr int R = PITCH * 2;  // row pitch in bytes
    lds_issue_tr8<0, 16 * R, 32, 16 * R + 32, 32 * R, 48 * R, 32 * R + 32, 48 * R + 32>(
        xt + (4 * lb + (lr >> 2)) * PITCH + 4 * (lr & 3), r);
}
__device__ __forceinline__ void take_x_frags(strd_s16x4 (&r)[8], bf16x8 (&xf)[2][2]) {
    lds_settle8(r);
    xf[0][0] = tr_pair(r[0], r[1]);
    xf[0][1] = tr_pair(r[2], r[3]);
    xf[1][0] = tr_pair(r[4], r[5]);
    xf[1][1] = tr_pair(r[6], r[7]);
}

// Output wave W of a workgroup: steps (a)-(d) for tokens 16W..16W+15 of every step.
template <int NS, int W, bool GATHER>
__device__ __forceinline__ void output_wave(Lds<NS> &lds, const float *__restrict__ D, bf16_t *__restrict__ y, int T,
                                            int H, int P, int h, int p0, int nsteps) {
    constexpr int KS = NS / 32;
    using L = Lds<NS>;
    const int lane = threadIdx.x & 63, lr = lane & 15, lb = lane >> 4;
    // The skip term D x_t rides on (c): D is added to the diagonal of the weights, M[t, t] += D (rounded to
    // bf16 with the weight, like every other term of the sum).
    const float Dh = D ? D[h] : 0.f;
    f32x4 dskip;
#pragma unroll
    for (int i = 0; i < 4; ++i) dskip[i] = 4 * lb + i == lr ? Dh : 0.f;
    const int tcol = 16 * W + lr;  // this lane's token inside the step
    bf16_t *yp = y + ((size_t)tcol * H + h) * P + p0 + 4 * lb;
    const size_t y_step = (size_t)kQ * H * P;
    // Operands that come from the B / C / x tiles alone are fetched one step early, in the tail
    // of the previous step when the LDS is quiet, and (a) is computed there too: carried from
    // step to step are c_t (for (d)), G^T and the x^T fragments of the coming step.
    bf16x8 cf[KS], xf[2][2];
    f32x4 acc[W + 1];
    strd_s16x4 xr8[8];
    bf16x8 bfr[W + 1][KS];
    // the LDS reads of the operands of step q: B and C fragments, then (separately, the registers
    // are free later) the x fragments
    auto fetch_issue_x = [&](int q) __attribute__((always_inline)) {
        issue_x_frags<L::kXP>(lds.xr[q % kXRing].x, lr, lb, xr8);
    };
    auto fetch_issue = [&](int q) __attribute__((always_inline)) {
        typename L::TileBC &tb = lds.bc[q % 3];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int jt = 0; jt <= W; ++jt)
                bfr[jt][ks] = *reinterpret_cast<const bf16x8 *>(&tb.b[(16 * jt + lr) * L::kCP + 32 * ks + 8 * lb]);
        // last: the products of (d) that are still queued read the current c fragments
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cf[ks] = *reinterpret_cast<const bf16x8 *>(&tb.c[tcol * L::kCP + 32 * ks + 8 * lb]);
        __builtin_amdgcn_sched_barrier(0);  // nothing moves across: loads above, arithmetic below
    };
    auto fetch_finish = [&]() __attribute__((always_inline)) {
        // (a): G^T tiles for key blocks jt <= W (independent accumulators)
#pragma unroll
        for (int jt = 0; jt <= W; ++jt) acc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int jt = 0; jt <= W; ++jt) acc[jt] = mfma16(bfr[jt][ks], cf[ks], acc[jt]);
        take_x_frags(xr8, xf);
    };

    if (GATHER) __syncthreads();  // the barriers of the prologue: (row tables written,)
    __syncthreads();              // first copies landed,
    fetch_issue(0);
    fetch_issue_x(0);
    fetch_finish();
    __syncthreads();              // scans of steps 0 and 1 published
    __syncthreads();              // (the state waves have read tile 0)

    for (int step = 0; step < nsteps; ++step) {
        const int cur = step & 1;
        typename L::Scan &bf = lds.scan[step % 3];
        // What depends on the previous step (scan, then state copy) is read here, all of it before
        // any arithmetic: after the barrier all waves hit the LDS at once and a round trip is long,
        // so the wave pays one, not one per phase.
        const float el_t = bf.ell[tcol];
        const float el_ref = bf.ell[W > 0 ? 16 * W - 1 : 0];
        f32x4 f_j[W > 0 ? W : 1];
#pragma unroll
        for (int jt = 0; jt < W; ++jt) f_j[jt] = *reinterpret_cast<const f32x4 *>(&bf.fw[L::fw_at(W) + 16 * jt + 4 * lb]);
        const f32x4 el_j = *reinterpret_cast<const f32x4 *>(&bf.ell[16 * W + 4 * lb]);
        const f32x4 dt_j = *reinterpret_cast<const f32x4 *>(&bf.dtv[16 * W + 4 * lb]);
        bf16x8 sf[2][KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                sf[pt][ks] = *reinterpret_cast<const bf16x8 *>(&lds.s[cur][16 * pt + lr][32 * ks + 8 * lb]);
        __builtin_amdgcn_sched_barrier(0);
        // (d): inter-step part from the state copy
        f32x4 yin[2];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            yin[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) yin[pt] = mfma16(sf[pt][ks], cf[ks], yin[pt]);
        }
        __builtin_amdgcn_sched_barrier(0);
        // The operands of the next step (its tiles were published by the barrier that ended the
        // previous step) are requested as soon as (d) has released the registers of the state
        // copy; their LDS round trip runs under (b), (c) and the stores.
        fetch_issue(step + 1);

        // (b): decay, dt and causal mask; pack pairs of key blocks as B operands of (c).
        // Blocks below the diagonal: 2^(l_t - l_j) dt_j = 2^(l_t - l_ref) * fw[j] with l_ref the scan
        // at the last token before this wave's block (both exponents <= 0); diagonal block: direct.
        bf16x4 m4[4];
        const float e_ref = W > 0 ? fast_exp2(el_t - el_ref) : 0.f;
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            m4[jt] = bf16x4{(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
            if (jt < W) {
#pragma unroll
                for (int i = 0; i < 4; ++i) m4[jt][i] = (bf16_t)(acc[jt < W ? jt : W][i] * e_ref * f_j[jt < W ? jt : 0][i]);
            } else if (jt == W) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float val = acc[W][i] * fast_exp2(el_t - el_j[i]) * dt_j[i] + dskip[i];
                    m4[jt][i] = (bf16_t)((4 * lb + i <= lr) ? val : 0.f);  // causal mask
                }
            }
        }
        // (c) intra-step part of Y^T[p, t]
        f32x4 yacc[2];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            yacc[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
                if (2 * pr <= W)
                    yacc[pt] = mfma16(xf[pr][pt],
                                      __builtin_shufflevector(m4[2 * pr], m4[2 * pr + 1], 0, 1, 2, 3, 4, 5, 6, 7), yacc[pt]);
        }
        const float carry = fast_exp2(el_t);
        __builtin_amdgcn_sched_barrier(0);
        fetch_issue_x(step + 1);  // (c) has released the x fragments of this step
        if (step * kQ + tcol < T) {
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                bf16x4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i) out[i] = (bf16_t)(yacc[pt][i] + carry * yin[pt][i]);
                *reinterpret_cast<bf16x4 *>(yp + 16 * pt) = out;
            }
        }
        yp += y_step;
        __builtin_amdgcn_sched_barrier(0);
        fetch_finish();
        lds_barrier();    // the y stores stay in flight
    }
}

// State wave SW: owns NT 16-row tiles of the state starting at tile T0 and does (e) for them.
template <int NS, int SW, bool GATHER>
__device__ __forceinline__ void state_wave(Lds<NS> &lds, const float *__restrict__ S_in, float *__restrict__ S_out,
                                           int P, int h, int p0, int nsteps) {
    using L = Lds<NS>;
    // state tiles per wave (n = 128: 2, 3, 2, 1 of 8 tiles; n = 64: one tile each): few where the
    // output wave on the same SIMD has much causal work (3), or where the helper wave runs (0)
    constexpr int NT = NS == 128 ? (SW == 1 ? 3 : SW == 3 ? 1 : 2) : 1;
    constexpr int T0 = NS == 128 ? (SW == 0 ? 0 : SW == 1 ? 2 : SW == 2 ? 5 : 7) : SW;
    const int lane = threadIdx.x & 63, lr = lane & 15, lb = lane >> 4;

    // state: fp32 master in registers ([n rows][p cols] tiles), bf16 copy in LDS
    f32x4 sacc[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            const int n0 = (T0 + nt) * 16 + lb * 4, pp = pt * 16 + lr;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (S_in) v = *reinterpret_cast<const f32x4 *>(S_in + ((size_t)h * P + p0 + pp) * NS + n0);
            sacc[nt][pt] = v;
            bf16x4 sv = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
            *reinterpret_cast<bf16x4 *>(&lds.s[0][pp][n0]) = sv;
        }
    // Operands of (e) for step q, all of them from tiles that were published a step or more before
    // q: b^T fragments of the owned state tiles ([tile][token half]) and the weighted x fragments
    // w_j x_j (token-contracted fragments of the x tile times the weights of the scan, rounded to
    // bf16).  They are prepared in the tail of step q - 1, so that a step starts with its products:
    // the new state is published early and no LDS round trip sits on the state's chain.
    bf16x8 bt[NT][2], xwf[2][2];
    float decay_q = 1.f;
    auto prepare = [&](int q) __attribute__((always_inline)) {
        typename L::TileBC &tb = lds.bc[q % 3];
        const typename L::Scan &m = lds.scan[q % 3];
        strd_s16x4 xr8[8], br8[(NT + 1) / 2][8];
        issue_x_frags<L::kXP>(lds.xr[q % kXRing].x, lr, lb, xr8);
#pragma unroll
        for (int n2 = 0; n2 < NT; n2 += 2) {  // two tiles per group of reads, the second only used if owned
            constexpr int R = L::kCP * 2;
            lds_issue_tr8<0, 16 * R, 32 * R, 48 * R, 32, 16 * R + 32, 32 * R + 32, 48 * R + 32>(
                &tb.b[(4 * lb + (lr >> 2)) * L::kCP + (T0 + n2) * 16 + 4 * (lr & 3)], br8[n2 / 2]);
        }
        // weights of the fragment's token slots: slot e is token 32 pr + 16 (e / 4) + 4 lb + e % 4
        f32x4 wv[2][2];
#pragma unroll
        for (int pr = 0; pr < 2; ++pr)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) wv[pr][hi] = *reinterpret_cast<const f32x4 *>(&m.w[32 * pr + 16 * hi + 4 * lb]);
        const float ell_q = m.ell[kQ - 1];
        bf16x8 xf[2][2];
        take_x_frags(xr8, xf);  // waits for the whole batch
#pragma unroll
        for (int n2 = 0; n2 < NT; n2 += 2) {
            lds_settle8(br8[n2 / 2]);
#pragma unroll
            for (int d = 0; d < 2; ++d)
                if (n2 + d < NT) {
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr)
                        bt[n2 + d][pr] = tr_pair(br8[n2 / 2][4 * d + 2 * pr], br8[n2 / 2][4 * d + 2 * pr + 1]);
                }
        }
        decay_q = fast_exp2(ell_q);
#pragma unroll
        for (int pr = 0; pr < 2; ++pr)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int e = 0; e < 8; ++e) xwf[pr][pt][e] = (bf16_t)((float)xf[pr][pt][e] * wv[pr][e >> 2][e & 3]);
    };

    // prologue, in step with the other waves: (row tables 0..3 |) first copies landed | scans 0
    // and 1
    if (GATHER) __syncthreads();
    __syncthreads();
    __syncthreads();
    prepare(0);
    // The first request of the copy waves' loop (tile 3) goes to the slot of tile 0: they wait here until
    // its b fragments have been read.  (Every later prepare(q) runs a step before tile q's slot is requested again.)
    __syncthreads();

    for (int step = 0; step < nsteps; ++step) {
        const int cur = step & 1;
        // (e) for the rows this wave owns: S^T = 2^(l_Q) S^T + b^T (w x)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] *= decay_q;
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] = mfma16(bt[nt][pr], xwf[pr][pt], sacc[nt][pt]);
        }
        // publish the new state copy
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                const f32x4 v = sacc[nt][pt];
                bf16x4 sv = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                *reinterpret_cast<bf16x4 *>(&lds.s[cur ^ 1][pt * 16 + lr][(T0 + nt) * 16 + lb * 4]) = sv;
            }
        __builtin_amdgcn_sched_barrier(0);
        prepare(step + 1);  // x, B and scan of step + 1 were published by the barrier that ended step - 1
        lds_barrier();
    }

    if (S_out) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                *reinterpret_cast<f32x4 *>(S_out + ((size_t)h * P + p0 + pt * 16 + lr) * NS + (T0 + nt) * 16 + lb * 4) =
                    sacc[nt][pt];
    }
}

// Helper wave: the copies of x and dt, and everything that is derived from dt alone, ahead of the
// steps that use it, so that no computing wave carries these LDS round trips: lane = token; the
// scan of dt*A, the key factors of (b) and the weights of (e) two steps ahead and, in gather mode,
// the source rows of the tokens five steps ahead.
template <int NS, bool GATHER>
__device__ __forceinline__ void helper_wave(Lds<NS> &lds, const bf16_t *__restrict__ x, const float *__restrict__ dt,
                                            const float *__restrict__ A, const int32_t *__restrict__ idx, int N, int K,
                                            int T, int H, int P, int h, int p0, int nsteps) {
    using L = Lds<NS>;
    using XT = typename L::XT;
    const int lane = threadIdx.x & 63;
    const float Al2 = A[h] * kLog2e;
    // a young wave of its SIMD, it would lose every issue arbitration against the two computing
    // waves there, and the copies it requests are the ones that come from furthest away
    __builtin_amdgcn_s_setprio(3);

    // gather mode: source rows of the tokens of `step`; tokens past T repeat the last one, and an
    // index outside [0, N) is clamped into the tensors instead of faulting.  Inside the loop the
    // entries of the kept-index list travel like every other input: an asynchronous copy into LDS
    // seven steps ahead, read two steps later and turned into the row table of five steps ahead --
    // a load into a register would make the wave wait for all its outstanding copies, too.
    const uint32_t last_row = (uint32_t)(N + (T - K) - 1);
    auto token_of = [&](int step) { return min(step * kQ + lane, T - 1); };
    auto row_of = [&](int step, int32_t kept) -> uint32_t {
        const int t = token_of(step);
        return min((uint32_t)(t < K ? kept : N + (t - K)), last_row);
    };
    auto kept_of = [&](int step) -> int32_t { return idx[min(token_of(step), K - 1)]; };  // K >= 1 here
    auto request_kept = [&](int step) __attribute__((always_inline)) {
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(idx + min(token_of(step), K - 1)),
            (__attribute__((address_space(3))) void *)lds.rawidx[step & 3], 4, 0, 0);
    };
    // scan of dt*A of `step` from the dt ring, the key factors of (b) and the weights of (e)
    auto make_scan = [&](int step, float raw) __attribute__((always_inline)) {
        const float dv = (step * kQ + lane < T) ? raw : 0.f;
        const float inc = wave_inclusive_scan_f32(dv * Al2);
        typename L::Scan &m = lds.scan[step % 3];
        m.ell[lane] = inc;
        m.dtv[lane] = dv;
        m.w[lane] = dv * fast_exp2(read_lane_f32(inc, kQ - 1) - inc);
#pragma unroll
        for (int wq = 1; wq < 4; ++wq) {  // only tokens j < 16 * wq are read; the exponent is <= 0 for them
            const float lref = read_lane_f32(inc, 16 * wq - 1);
            if (lane < 16 * wq) m.fw[L::fw_at(wq) + lane] = dv * fast_exp2(lref - inc);
        }
    };

    // The asynchronous global -> LDS copies of x (three steps ahead, ring of 4) and dt (four steps
    // ahead, ring of 5).  Byte offsets (32 bits) of this lane's copies at the next step to request,
    // per-step strides and end-of-sequence clamps (rows past T re-read the last row; dt = 0 makes
    // them inert); gather mode: (row in the step, column offset) per copy, the row itself comes
    // from the row table.
    const uint32_t x_row = (uint32_t)H * P * 2, dt_row = (uint32_t)H * 4;
    uint32_t off_x[XT::kIssues], lim_x[XT::kIssues];
    int row_x[XT::kIssues];
    uint32_t off_dt = (uint32_t)lane * dt_row + (uint32_t)h * 4;
    const uint32_t lim_dt = (uint32_t)(T - 1) * dt_row + (uint32_t)h * 4;
    int next_x = 0, next_dt = 0;
#pragma unroll
    for (int i = 0; i < XT::kIssues; ++i) {
        int cv;
        XT::slot(0, lane, i, row_x[i], cv);
        const uint32_t col = ((uint32_t)h * P + p0 + cv * 8) * 2;
        off_x[i] = GATHER ? col : (uint32_t)row_x[i] * x_row + col;
        lim_x[i] = (uint32_t)(T - 1) * x_row + col;
    }
    // each call requests the next not yet requested step of its stream into ring slot b
    auto request_x = [&](int b) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < XT::kIssues; ++i) {
            const uint32_t o = GATHER ? lds.rowtab[next_x & 3][row_x[i]] * x_row + off_x[i] : min(off_x[i], lim_x[i]);
            XT::issue(reinterpret_cast<const char *>(x) + o, lds.xr[b].x, 0, i);
            if (!GATHER) off_x[i] += kQ * x_row;
        }
        ++next_x;
    };
    auto request_dt = [&](int b) __attribute__((always_inline)) {  // 64 lanes x 4 bytes
        const uint32_t o = GATHER ? lds.rowtab[next_dt & 3][lane] * dt_row + (uint32_t)h * 4 : min(off_dt, lim_dt);
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(reinterpret_cast<const char *>(dt) + o),
            (__attribute__((address_space(3))) void *)lds.dt[b], 4, 0, 0);
        off_dt += kQ * dt_row;
        ++next_dt;
    };
    // Copies issued per step (x, dt and, in gather mode, the entries of the kept-index list);
    // everything older has landed once at most that many are outstanding (they complete in order).  s_waitcnt immediate, gfx9 layout:
    // vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
    constexpr int kNewest = XT::kIssues + 1 + (GATHER ? 1 : 0);
    constexpr int kWaitOlder = (kNewest & 15) | (7 << 4) | (15 << 8) | ((kNewest >> 4) << 14);

    // prologue, in step with the other waves: (row tables 0..3 |) first copies landed | scans 0
    // and 1 (, row table 4)
    if (GATHER) {
#pragma unroll
        for (int q = 0; q < 4; ++q) lds.rowtab[q][lane] = row_of(q, kept_of(q));
        lds.rawidx[5 & 3][lane] = kept_of(5);  // read in steps 0 and 1, before the first copied entries
        lds.rawidx[6 & 3][lane] = kept_of(6);
        __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {  // fill the rings up to their look-ahead (x: steps 0..2, dt: steps 0..3)
        if (q < 3) request_x(q);
        request_dt(q);
    }
    async_tile_wait();
    __syncthreads();
    if (GATHER) lds.rowtab[0][lane] = row_of(4, kept_of(4));  // the prologue's requests have read table 0
    make_scan(0, lds.dt[0][lane]);
    make_scan(1, lds.dt[1][lane]);
    __syncthreads();
    __syncthreads();  // (the state waves have read tile 0)

    for (int step = 0; step < nsteps; ++step) {
        const bool more = step + 3 < nsteps;  // uniform; nothing past the last step is requested
        // dt up to step + 2 landed before the barrier that ended the previous step; read before this
        // step's copies are requested, so that no wait for them can sit in front of the read
        const float raw = lds.dt[(step + 2) % kDtRing][lane];
        int32_t kept = 0;
        if (GATHER) kept = lds.rawidx[(step + 5) & 3][lane];  // requested in step - 2 (or by the prologue)
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            request_x((step + kXRing - 1) % kXRing);     // x of step + 3; slot last read in step - 1
            request_dt((step + kDtRing - 1) % kDtRing);  // dt of step + 4; slot last read in step - 2
            if (GATHER) request_kept(step + 7);          // slot last read in step - 2
        }
        make_scan(step + 2, raw);
        // gather mode: rows of step + 5, first used in the next step (dt of step + 5); the slot held
        // the rows of step + 1, last used two steps ago
        if (GATHER) lds.rowtab[(step + 1) & 3][lane] = row_of(step + 5, kept);
        if (more)
            __builtin_amdgcn_s_waitcnt(kWaitOlder);  // everything requested in earlier steps has landed
        else
            async_tile_wait();
        lds_barrier();  // publishes it; this step's copies stay in flight
    }
}

// Copy waves: the B and C tiles reach LDS through their asynchronous global -> LDS copies, half a
// tile each.  They run ahead of the consumers by a fixed number of steps and block on the copy
// path instead of them.
// GATHER: token t of the sequence is row idx[t] (t < K) or N + t - K of the tensors, i.e. the
// kernel reads the uncompacted x, dt, B, C through the kept-index list instead of a compacted copy;
// the rows of a step come from a table that the helper wave keeps five steps ahead.
template <int NS, int CW, bool GATHER>
__device__ __forceinline__ void copy_wave(Lds<NS> &lds, const bf16_t *__restrict__ B, const bf16_t *__restrict__ C,
                                          int T, int G, int g, int nsteps) {
    using L = Lds<NS>;
    using BC = typename L::BC;
    const int lane = threadIdx.x & 63;
    // Byte offsets (32 bits) of this lane's copies at the next step to request, per-step strides and
    // end-of-sequence clamps (rows past T re-read the last row; dt = 0 makes them inert).
    const uint32_t bc_row = (uint32_t)G * NS * 2;
    // dense mode: running offsets; gather mode: (row in the step, column offset) per copy and the
    // number of the next step to request, the row itself comes from the row table
    uint32_t off_bc[BC::kIssues], lim_bc[BC::kIssues];
    int row_bc[BC::kIssues];
    int next_bc = 0;
#pragma unroll
    for (int i = 0; i < BC::kIssues; ++i) {
        int cv;
        BC::slot(CW, lane, i, row_bc[i], cv);
        const uint32_t col = ((uint32_t)g * NS + cv * 8) * 2;
        off_bc[i] = GATHER ? col : (uint32_t)row_bc[i] * bc_row + col;
        lim_bc[i] = (uint32_t)(T - 1) * bc_row + col;
    }
    // each call requests the next not yet requested step of its stream into ring slot b
    auto request_bc = [&](int b) {
#pragma unroll
        for (int i = 0; i < BC::kIssues; ++i) {
            const uint32_t o = GATHER ? lds.rowtab[next_bc & 3][row_bc[i]] * bc_row + off_bc[i] : min(off_bc[i], lim_bc[i]);
            BC::issue(reinterpret_cast<const char *>(C) + o, lds.bc[b].c, CW, i);
            BC::issue(reinterpret_cast<const char *>(B) + o, lds.bc[b].b, CW, i);
            if (!GATHER) off_bc[i] += kQ * bc_row;
        }
        ++next_bc;
    };
    // Copies issued per step; everything older has landed once at most that many are outstanding
    // (vector-memory operations complete in order).  s_waitcnt immediate, gfx9 layout:
    // vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
    constexpr int kNewest = 2 * BC::kIssues;
    static_assert(kNewest < 64, "vmcnt has 6 bits");
    constexpr int kWaitOlder = (kNewest & 15) | (7 << 4) | (15 << 8) | ((kNewest >> 4) << 14);

    // prologue: fill the ring up to its look-ahead (steps 0..2)
    if (GATHER) __syncthreads();  // row tables of steps 0..3 written
#pragma unroll
    for (int q = 0; q < 3; ++q) request_bc(q);
    async_tile_wait();
    __syncthreads();  // first copies landed
    __syncthreads();  // (scans of steps 0 and 1)
    __syncthreads();  // the state waves have read tile 0 (the first request of the loop overwrites it)

    for (int step = 0; step < nsteps; ++step) {
        if (step + 3 < nsteps) {  // uniform; nothing past the last step is requested
            request_bc(step % 3);                    // tile step + 3; the slot's tile (step) was read in step - 1
            __builtin_amdgcn_s_waitcnt(kWaitOlder);  // everything requested in earlier steps has landed
        } else {
            async_tile_wait();
        }
        lds_barrier();  // publishes it; this step's copies stay in flight
    }
}

template <int NS, bool GATHER>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 3))) void ssd_mfma_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ dt, const float *__restrict__ A,
    const bf16_t *__restrict__ B, const bf16_t *__restrict__ C, const float *__restrict__ D,
    const float *__restrict__ S_in, bf16_t *__restrict__ y, float *__restrict__ S_out,
    const int32_t *__restrict__ idx, int N, int K, int T, int H, int P, int G, int nunits) {
    using L = Lds<NS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    L &lds = *reinterpret_cast<L *>(smem_raw);

    const int unit = xcd_swizzle(blockIdx.x, nunits);
    if (unit >= nunits) return;
    const int nslab = P / kPB;
    const int h = unit / nslab, p0 = (unit % nslab) * kPB, g = h / (H / G);
    const int nsteps = (T + kQ - 1) / kQ;
    switch (threadIdx.x >> 6) {
        case 0: output_wave<NS, 0, GATHER>(lds, D, y, T, H, P, h, p0, nsteps); break;
        case 1: output_wave<NS, 1, GATHER>(lds, D, y, T, H, P, h, p0, nsteps); break;
        case 2: output_wave<NS, 2, GATHER>(lds, D, y, T, H, P, h, p0, nsteps); break;
        case 3: output_wave<NS, 3, GATHER>(lds, D, y, T, H, P, h, p0, nsteps); break;
        case 4: state_wave<NS, 0, GATHER>(lds, S_in, S_out, P, h, p0, nsteps); break;
        case 5: state_wave<NS, 1, GATHER>(lds, S_in, S_out, P, h, p0, nsteps); break;
        case 6: state_wave<NS, 2, GATHER>(lds, S_in, S_out, P, h, p0, nsteps); break;
        case 7: state_wave<NS, 3, GATHER>(lds, S_in, S_out, P, h, p0, nsteps); break;
        // wave i runs on SIMD i % 4: the helper shares a SIMD with the lightest output wave, the
        // heaviest output wave (3) shares its SIMD with the lightest state wave only
        case 8: helper_wave<NS, GATHER>(lds, x, dt, A, idx, N, K, T, H, P, h, p0, nsteps); break;
        case 9: copy_wave<NS, 0, GATHER>(lds, B, C, T, G, g, nsteps); break;
        case 10: copy_wave<NS, 1, GATHER>(lds, B, C, T, G, g, nsteps); break;
        default: copy_wave<NS, 2, GATHER>(lds, B, C, T, G, g, nsteps); break;
    }
}

template <int NS, bool GATHER>
int launch(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
           const float *S_in, void *y, float *S_out, const int32_t *idx, int N, int K, int T, int H, int P, int G,
           hipStream_t st) {
    const int nunits = H * (P / kPB);
    const size_t smem = sizeof(Lds<NS>);
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&ssd_mfma_kernel<NS, GATHER>), smem))
        return STRD_EHIP;
    ssd_mfma_kernel<NS, GATHER><<<xcd_grid(nunits), kThreads, smem, st>>>(
        (const bf16_t *)x, dt, A, (const bf16_t *)B, (const bf16_t *)C, D, S_in, (bf16_t *)y, S_out, idx, N, K, T, H, P,
        G, nunits);
    return launch_status();
}

}  // namespace

// `rows` = number of rows of the source tensors (T for the dense call, N + M for the gather call)
bool ssd_mfma_supported(int T, int rows, int H, int P, int G, int n, strd_dtype io) {
    // staging uses 32-bit byte offsets from the tensor bases
    const unsigned long long lim = 1ull << 32, r = (unsigned long long)(rows > T ? rows : T) + 2 * kQ;
    return io == STRD_BF16 && T >= 1 && (n == 64 || n == 128) && P % kPB == 0 &&
           (long long)H * (P / kPB) < (1 << 24) && r * H * P * 2 < lim && r * G * n * 2 < lim && r * H * 4 < lim;
}

int ssd_mfma(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
             const float *S_in, void *y, float *S_out, const int32_t *idx, int N, int K, int T, int H, int P, int G,
             int n, hipStream_t st) {
    if (idx) {
        if (n == 128) return launch<128, true>(x, dt, A, B, C, D, S_in, y, S_out, idx, N, K, T, H, P, G, st);
        if (n == 64) return launch<64, true>(x, dt, A, B, C, D, S_in, y, S_out, idx, N, K, T, H, P, G, st);
    } else {
        if (n == 128) return launch<128, false>(x, dt, A, B, C, D, S_in, y, S_out, nullptr, 0, 0, T, H, P, G, st);
        if (n == 64) return launch<64, false>(x, dt, A, B, C, D, S_in, y, S_out, nullptr, 0, 0, T, H, P, G, st);
    }
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
