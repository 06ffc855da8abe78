// ssd_prefill on bf16 matrix cores: the Mamba-2 recurrence (paper Eqs. "ssm_state_update",
// "ssm_output") in its chunked form, i.e. the unrolled sum (Eq. "ssm_unrolled") split at
// 64-token boundaries, with the recurrent state kept in registers for the whole sequence.
//
// Decomposition.  One workgroup (8 waves) owns one head h and a slab of 32 of its P channels
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
// step.  Waves 4-7 ("state waves") each own a quarter of the state rows for (e), and between
// them stage the next step's tiles global -> registers -> LDS, including the weighted copy
// w_j x_j and the scan of dt*A.  The two roles share each SIMD, so the state waves' memory
// latency hides behind the output waves' arithmetic.  LDS tiles and the bf16 state copy are
// double-buffered: one workgroup barrier per step.  Rows past T are staged as copies of the
// last row with dt = 0, which makes them inert in (b)-(e); their y rows are not stored.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kQ = 64;         // tokens per step
constexpr int kPB = 32;        // channels of the head per workgroup
constexpr int kThreads = 512;  // 4 output waves + 4 state waves
constexpr int kStage = 256;    // threads that stage tiles (the state waves)
constexpr int kXPitch = 48;    // bf16 elements per row of the x tiles (32 used)
constexpr float kLog2e = 1.4426950408889634f;

template <int NS>
struct Lds {
    static constexpr int kCP = NS + 16;  // bf16 elements per row of the B / C tiles
    static constexpr int kSP = NS + 8;   // bf16 elements per row of the state copy
    struct Buf {
        bf16_t c[kQ][kCP];
        bf16_t b[kQ][kCP];
        bf16_t x[kQ][kXPitch];
        bf16_t xw[kQ][kXPitch];  // w_j * x_j
        float ell[kQ];           // inclusive cumulative sum of dt*A*log2(e) inside the step
        float dtv[kQ];           // dt (0 past the end of the sequence)
    };
    Buf buf[2];
    bf16_t s[2][kPB][kSP];  // state before the step, [p][n]
};

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Transposing LDS read.  Within each group of 16 lanes, lane r must pass the address of
// element [k0 + r/4][c0 + 4*(r%4)] of a row-major bf16 tile; it receives [k0..k0+3][c0 + r].
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t *p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
    return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 cat(bf16x4 lo, bf16x4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

__device__ __forceinline__ uint4 ld16(const void *base, uint32_t byte_off) {
    return *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Output wave W of a workgroup: steps (a)-(d) for tokens 16W..16W+15 of every step.
template <int NS, int W>
__device__ __forceinline__ void output_wave(Lds<NS> &lds, const float *__restrict__ D, bf16_t *__restrict__ y, int T,
                                            int H, int P, int h, int p0, int nsteps) {
    constexpr int KS = NS / 32;
    using L = Lds<NS>;
    const int lane = threadIdx.x & 63, lr = lane & 15, lb = lane >> 4;
    const float Dh = D ? D[h] : 0.f;
    const int tcol = 16 * W + lr;  // this lane's token inside the step
    bf16_t *yp = y + ((size_t)tcol * H + h) * P + p0 + 4 * lb;
    const size_t y_step = (size_t)kQ * H * P;
    __syncthreads();  // pairs with the state waves' barrier after the first commit

    for (int step = 0; step < nsteps; ++step) {
        const int cur = step & 1;
        typename L::Buf &bf = lds.buf[cur];
        const float el_t = bf.ell[tcol];

        // c_t fragments: B operand of (a) and of (d)
        bf16x8 cf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cf[ks] = *reinterpret_cast<const bf16x8 *>(&bf.c[tcol][32 * ks + 8 * lb]);

        // (a): G^T tiles for key blocks jt <= W (independent accumulators)
        f32x4 acc[W + 1];
#pragma unroll
        for (int jt = 0; jt <= W; ++jt) acc[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int jt = 0; jt <= W; ++jt) {
                const bf16x8 bfr = *reinterpret_cast<const bf16x8 *>(&bf.b[16 * jt + lr][32 * ks + 8 * lb]);
                acc[jt] = mfma16(bfr, cf[ks], acc[jt]);
            }
        // (b): decay, dt and causal mask; pack pairs of key blocks as B operands of (c)
        bf16x4 m4[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            m4[jt] = bf16x4{(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
            if (jt <= W) {
                const f32x4 el_j = *reinterpret_cast<const f32x4 *>(&bf.ell[16 * jt + 4 * lb]);
                const f32x4 dt_j = *reinterpret_cast<const f32x4 *>(&bf.dtv[16 * jt + 4 * lb]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float val = acc[jt < W ? jt : W][i] * fast_exp2(el_t - el_j[i]) * dt_j[i];
                    // only the diagonal block needs the causal mask
                    m4[jt][i] = (bf16_t)((jt < W || 4 * lb + i <= lr) ? val : 0.f);
                }
            }
        }

        // (c) intra-step part and (d) carried-state part of Y^T[p, t]
        f32x4 yacc[2], yin[2];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            yacc[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
            yin[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
                if (2 * pr <= W) {
                    // token slots of a fragment: s < 4 is token 32*pr + 4*lb + s, s >= 4 adds 16
                    const bf16_t *a0 = &bf.x[32 * pr + 4 * lb + (lr >> 2)][16 * pt + 4 * (lr & 3)];
                    const bf16x8 xf = cat(lds_read_tr(a0), lds_read_tr(a0 + 16 * kXPitch));
                    yacc[pt] = mfma16(xf, cat(m4[2 * pr], m4[2 * pr + 1]), yacc[pt]);
                }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 sf = *reinterpret_cast<const bf16x8 *>(&lds.s[cur][16 * pt + lr][32 * ks + 8 * lb]);
                yin[pt] = mfma16(sf, cf[ks], yin[pt]);
            }
        }
        const float carry = fast_exp2(el_t);
        if (step * kQ + tcol < T) {
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                bf16x4 out;
                if (D) {
                    const bf16x4 xv = *reinterpret_cast<const bf16x4 *>(&bf.x[tcol][16 * pt + 4 * lb]);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        out[i] = (bf16_t)(yacc[pt][i] + carry * yin[pt][i] + Dh * (float)xv[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) out[i] = (bf16_t)(yacc[pt][i] + carry * yin[pt][i]);
                }
                *reinterpret_cast<bf16x4 *>(yp + 16 * pt) = out;
            }
        }
        yp += y_step;
        __syncthreads();
    }
}

template <int NS>
__global__ __launch_bounds__(kThreads) void ssd_mfma_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ dt, const float *__restrict__ A,
    const bf16_t *__restrict__ B, const bf16_t *__restrict__ C, const float *__restrict__ D,
    const float *__restrict__ S_in, bf16_t *__restrict__ y, float *__restrict__ S_out, int T, int H, int P, int G,
    int nunits) {
    constexpr int KS = NS / 32;            // k-steps over the state dimension
    constexpr int NT = NS / 64;            // 16-row state tiles owned by one state wave
    constexpr int VR = NS / 8;             // 16-byte vectors per B / C row
    constexpr int VPT = kQ * VR / kStage;  // B (or C) vectors staged per staging thread
    using L = Lds<NS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    L &lds = *reinterpret_cast<L *>(smem_raw);

    const int unit = xcd_swizzle(blockIdx.x, nunits);
    if (unit >= nunits) return;
    const int nslab = P / kPB;
    const int h = unit / nslab, p0 = (unit % nslab) * kPB, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lr = lane & 15, lb = lane >> 4;
    const int nsteps = (T + kQ - 1) / kQ;

    if (w >= 4) {
        // =========================== state waves ===========================================
        const int sw = w - 4, st = tid - kStage;
        const int nbase = sw * (NS / 4);  // first state row of this wave
        const float Al2 = A[h] * kLog2e;

        // byte offsets of this thread's staging vectors at step 0, their per-step stride and
        // their value at the last row of the sequence (rows past T re-read that row)
        const uint32_t bc_row = (uint32_t)G * NS * 2, x_row = (uint32_t)H * P * 2, dt_row = (uint32_t)H * 4;
        uint32_t off_bc[VPT], lim_bc[VPT];
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int v = st + i * kStage, r = v / VR, cv = v % VR;
            const uint32_t col = ((uint32_t)g * NS + cv * 8) * 2;
            off_bc[i] = (uint32_t)r * bc_row + col;
            lim_bc[i] = (uint32_t)(T - 1) * bc_row + col;
        }
        const uint32_t x_col = ((uint32_t)h * P + p0 + (st & 3) * 8) * 2;
        uint32_t off_x = (uint32_t)(st >> 2) * x_row + x_col;
        const uint32_t lim_x = (uint32_t)(T - 1) * x_row + x_col;
        uint32_t off_dt = (uint32_t)lane * dt_row + (uint32_t)h * 4;
        const uint32_t lim_dt = (uint32_t)(T - 1) * dt_row + (uint32_t)h * 4;

        // two register sets: a step's tiles are requested two steps before they are needed
        struct Regs {
            uint4 pc[VPT], pb[VPT], px;
            float pdt;
        };
        auto prefetch = [&](Regs &rg, int step) {
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                const uint32_t o = min(off_bc[i], lim_bc[i]);
                rg.pc[i] = ld16(C, o);
                rg.pb[i] = ld16(B, o);
                off_bc[i] += kQ * bc_row;
            }
            rg.px = ld16(x, min(off_x, lim_x));
            off_x += kQ * x_row;
            const float dv = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(dt) + min(off_dt, lim_dt));
            rg.pdt = (step * kQ + lane < T) ? dv : 0.f;
            off_dt += kQ * dt_row;
        };
        auto commit = [&](const Regs &rg, int b) {
            typename L::Buf &bf = lds.buf[b];
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                const int v = st + i * kStage, r = v / VR, cv = v % VR;
                *reinterpret_cast<uint4 *>(&bf.c[r][cv * 8]) = rg.pc[i];
                *reinterpret_cast<uint4 *>(&bf.b[r][cv * 8]) = rg.pb[i];
            }
            // scan of dt*A over the step (every state wave does it: lane = token)
            float inc = rg.pdt * Al2;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const float up = __shfl_up(inc, o, kWave);
                if (lane >= o) inc += up;
            }
            const float lq = __shfl(inc, kWave - 1, kWave);
            const float wv = rg.pdt * fast_exp2(lq - inc);
            if (sw == 0) {
                bf.ell[lane] = inc;
                bf.dtv[lane] = rg.pdt;
            }
            // x tile and its weighted copy; this thread holds 8 channels of row st / 4
            const float wrow = __shfl(wv, 16 * sw + (lane >> 2), kWave);
            const bf16x8 xv = __builtin_bit_cast(bf16x8, rg.px);
            bf16x8 xs;
#pragma unroll
            for (int e = 0; e < 8; ++e) xs[e] = (bf16_t)((float)xv[e] * wrow);
            *reinterpret_cast<uint4 *>(&bf.x[st >> 2][(st & 3) * 8]) = rg.px;
            *reinterpret_cast<bf16x8 *>(&bf.xw[st >> 2][(st & 3) * 8]) = xs;
        };
        Regs ra, rb;

        // state: fp32 master in registers ([n rows][p cols] tiles), bf16 copy in LDS
        f32x4 sacc[NT][2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                const int n0 = nbase + nt * 16 + lb * 4, pp = pt * 16 + lr;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (S_in) v = *reinterpret_cast<const f32x4 *>(S_in + ((size_t)h * P + p0 + pp) * NS + n0);
                sacc[nt][pt] = v;
                bf16x4 sv = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                *reinterpret_cast<bf16x4 *>(&lds.s[0][pp][n0]) = sv;
            }
        // prefetches past the end re-read the last row (offsets are clamped) and are never
        // consumed, so the loop body has no conditional loads or LDS writes
        prefetch(ra, 0);
        commit(ra, 0);
        prefetch(ra, 1);
        __syncthreads();

        // one step; `held` carries the tiles of step + 1, `next` receives those of step + 2
        auto do_step = [&](int step, Regs &held, Regs &next) {
            const int cur = step & 1;
            typename L::Buf &bf = lds.buf[cur];
            prefetch(next, step + 2);

            // (e): token slots of a fragment: s < 4 is token 32*pr + 4*lb + s, s >= 4 adds 16
            const float decay_q = fast_exp2(bf.ell[kQ - 1]);
            bf16x8 xf[2][2];
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const bf16_t *a0 = &bf.xw[32 * pr + 4 * lb + (lr >> 2)][16 * pt + 4 * (lr & 3)];
                    xf[pr][pt] = cat(lds_read_tr(a0), lds_read_tr(a0 + 16 * kXPitch));
                }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] *= decay_q;
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    const bf16_t *a0 = &bf.b[32 * pr + 4 * lb + (lr >> 2)][nbase + 16 * nt + 4 * (lr & 3)];
                    const bf16x8 bt = cat(lds_read_tr(a0), lds_read_tr(a0 + 16 * L::kCP));
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] = mfma16(bt, xf[pr][pt], sacc[nt][pt]);
                }
            }
            // publish the new state copy and the next step's tiles into the other buffers
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const f32x4 v = sacc[nt][pt];
                    bf16x4 sv = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
                    *reinterpret_cast<bf16x4 *>(&lds.s[cur ^ 1][pt * 16 + lr][nbase + nt * 16 + lb * 4]) = sv;
                }
            commit(held, cur ^ 1);
            __syncthreads();
        };
        for (int step = 0; step < nsteps; step += 2) {
            do_step(step, ra, rb);
            if (step + 1 < nsteps) do_step(step + 1, rb, ra);
        }

        if (S_out) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int pt = 0; pt < 2; ++pt)
                    *reinterpret_cast<f32x4 *>(S_out + ((size_t)h * P + p0 + pt * 16 + lr) * NS + nbase + nt * 16 +
                                               lb * 4) = sacc[nt][pt];
        }
    } else {
        // =========================== output waves ==========================================
        // one straight-line specialisation per wave, so that the causal trip counts are
        // compile-time constants and the independent MFMA chains can be interleaved
        switch (w) {
            case 0: output_wave<NS, 0>(lds, D, y, T, H, P, h, p0, nsteps); break;
            case 1: output_wave<NS, 1>(lds, D, y, T, H, P, h, p0, nsteps); break;
            case 2: output_wave<NS, 2>(lds, D, y, T, H, P, h, p0, nsteps); break;
            default: output_wave<NS, 3>(lds, D, y, T, H, P, h, p0, nsteps); break;
        }
    }
}

template <int NS>
int launch(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
           const float *S_in, void *y, float *S_out, int T, int H, int P, int G, hipStream_t st) {
    const int nunits = H * (P / kPB);
    const size_t smem = sizeof(Lds<NS>);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&ssd_mfma_kernel<NS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return STRD_EHIP;
        configured = true;
    }
    ssd_mfma_kernel<NS><<<xcd_grid(nunits), kThreads, smem, st>>>(
        (const bf16_t *)x, dt, A, (const bf16_t *)B, (const bf16_t *)C, D, S_in, (bf16_t *)y, S_out, T, H, P, G,
        nunits);
    return launch_status();
}

}  // namespace

bool ssd_mfma_supported(int T, int H, int P, int G, int n, strd_dtype io) {
    // staging uses 32-bit byte offsets from the tensor bases
    const unsigned long long lim = 1ull << 32;
    return io == STRD_BF16 && T >= 1 && (n == 64 || n == 128) && P % kPB == 0 &&
           (long long)H * (P / kPB) < (1 << 24) && (unsigned long long)(T + kQ) * H * P * 2 < lim &&
           (unsigned long long)(T + kQ) * G * n * 2 < lim && (unsigned long long)(T + kQ) * H * 4 < lim;
}

int ssd_mfma(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
             const float *S_in, void *y, float *S_out, int T, int H, int P, int G, int n, hipStream_t st) {
    if (n == 128) return launch<128>(x, dt, A, B, C, D, S_in, y, S_out, T, H, P, G, st);
    if (n == 64) return launch<64>(x, dt, A, B, C, D, S_in, y, S_out, T, H, P, G, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
