// ssd_prefill on bf16 matrix cores: the Mamba-2 recurrence (paper Eqs. "ssm_state_update",
// "ssm_output") in its chunked form, i.e. the unrolled sum (Eq. "ssm_unrolled") split at
// 64-token boundaries, with the recurrent state kept in registers for the whole sequence.
//
// Decomposition.  One workgroup (4 waves) owns one head h and a slab of 32 of its P channels
// and walks the sequence in 64-token steps; nothing but x, dt, B, C is read from HBM and
// nothing but y (and the final state) is written.  Per step, with l_t the in-step cumulative
// sum of dt*A (in log2 units) and all tiles staged in LDS:
//   (a) G^T[j,t] = b_j . c_t                        MFMA, contraction over the state dim n
//   (b) M^T[j,t] = G^T[j,t] * 2^(l_t-l_j) * dt_j  for j <= t, else 0     (fp32, then bf16)
//   (c) Y^T[p,t] = sum_j x_j[p] M^T[j,t]             MFMA, contraction over tokens
//   (d) Y^T[p,t] += 2^(l_t) * sum_n S[p,n] c_t[n]    MFMA, S = state before the step (bf16 copy)
//   (e) S^T[n,p] = 2^(l_Q) S^T[n,p] + sum_j (w_j b_j[n]) x_j[p],  w_j = dt_j 2^(l_Q-l_j)   MFMA
// Every MFMA is v_mfma_f32_16x16x32_bf16.  Results are kept "token on the lane" (columns of
// the accumulator tiles are tokens) so every token-dependent factor is one scalar per lane.
// Operands whose contraction index is the token (x and b in (c), (e)) are read from their
// token-major LDS tiles with the transposing LDS read (ds_read_b64_tr_b16).
//
// Wave w of the workgroup computes (a)-(d) for tokens 16w..16w+15 of the step and owns rows
// n/4*w .. of the state for (e).  LDS tiles and the bf16 state copy are double-buffered so a
// step needs a single workgroup barrier; the next step's tiles are prefetched into registers
// while the current one is computed.  Rows past T are staged as zeros with dt = 0, which makes
// them inert in (b)-(e); their y rows are not stored.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kQ = 64;         // tokens per step
constexpr int kPB = 32;        // channels of the head per workgroup
constexpr int kThreads = 256;  // 4 waves
constexpr int kXPitch = 48;    // bf16 elements per row of the x tile (32 used)
constexpr float kLog2e = 1.4426950408889634f;

template <int NS>
struct Lds {
    static constexpr int kCP = NS + 16;  // bf16 elements per row of the B / C tiles
    static constexpr int kSP = NS + 8;   // bf16 elements per row of the state copy
    struct Buf {
        bf16_t c[kQ][kCP];
        bf16_t b[kQ][kCP];
        bf16_t x[kQ][kXPitch];
        float ell[kQ];  // inclusive cumulative sum of dt*A*log2(e) inside the step
        float dtv[kQ];  // dt (0 past the end of the sequence)
        float wv[kQ];   // dt_j * 2^(l_Q - l_j)
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

template <int NS>
__global__ __launch_bounds__(kThreads) void ssd_mfma_kernel(
    const bf16_t *__restrict__ x, const float *__restrict__ dt, const float *__restrict__ A,
    const bf16_t *__restrict__ B, const bf16_t *__restrict__ C, const float *__restrict__ D,
    const float *__restrict__ S_in, bf16_t *__restrict__ y, float *__restrict__ S_out, int T, int H, int P, int G,
    int nunits) {
    constexpr int KS = NS / 32;       // k-steps over the state dimension
    constexpr int NT = NS / 64;       // 16-row state tiles owned by one wave
    constexpr int VR = NS / 8;        // 16-byte vectors per B / C row
    constexpr int VPT = kQ * VR / kThreads;  // B (or C) vectors staged per thread
    using L = Lds<NS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    L &lds = *reinterpret_cast<L *>(smem_raw);

    const int unit = xcd_swizzle(blockIdx.x, nunits);
    if (unit >= nunits) return;
    const int nslab = P / kPB;
    const int h = unit / nslab, p0 = (unit % nslab) * kPB, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lr = lane & 15, lb = lane >> 4;
    const int nsteps = (T + kQ - 1) / kQ;
    const float Al2 = A[h] * kLog2e;
    const float Dh = D ? D[h] : 0.f;
    const int nbase = w * (NS / 4);   // first state row of this wave

    // ---- staging: global -> registers -> LDS --------------------------------------------
    uint4 pc[VPT], pb[VPT], px;
    float pdt = 0.f;
    auto prefetch = [&](int step) {
        const int t0 = step * kQ;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int v = tid + i * kThreads, r = v / VR, cv = v % VR;
            const bool in = t0 + r < T;
            const size_t off = ((size_t)(t0 + r) * G + g) * NS + cv * 8;
            pc[i] = in ? *reinterpret_cast<const uint4 *>(C + off) : make_uint4(0, 0, 0, 0);
            pb[i] = in ? *reinterpret_cast<const uint4 *>(B + off) : make_uint4(0, 0, 0, 0);
        }
        {
            const int r = tid >> 2, cv = tid & 3;
            const bool in = t0 + r < T;
            px = in ? *reinterpret_cast<const uint4 *>(x + ((size_t)(t0 + r) * H + h) * P + p0 + cv * 8)
                    : make_uint4(0, 0, 0, 0);
        }
        if (w == 0) pdt = (t0 + lane < T) ? dt[(size_t)(t0 + lane) * H + h] : 0.f;
    };
    auto commit = [&](int b) {
        typename L::Buf &bf = lds.buf[b];
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int v = tid + i * kThreads, r = v / VR, cv = v % VR;
            *reinterpret_cast<uint4 *>(&bf.c[r][cv * 8]) = pc[i];
            *reinterpret_cast<uint4 *>(&bf.b[r][cv * 8]) = pb[i];
        }
        *reinterpret_cast<uint4 *>(&bf.x[tid >> 2][(tid & 3) * 8]) = px;
        if (w == 0) {
            float inc = pdt * Al2;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const float up = __shfl_up(inc, o, kWave);
                if (lane >= o) inc += up;
            }
            const float lq = __shfl(inc, kWave - 1, kWave);
            bf.ell[lane] = inc;
            bf.dtv[lane] = pdt;
            bf.wv[lane] = pdt * fast_exp2(lq - inc);
        }
    };

    // ---- state: fp32 master in registers ([n rows][p cols] tiles), bf16 copy in LDS -------
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
    if (nsteps > 0) {
        prefetch(0);
        commit(0);
    }
    __syncthreads();

    for (int step = 0; step < nsteps; ++step) {
        const int cur = step & 1;
        typename L::Buf &bf = lds.buf[cur];
        if (step + 1 < nsteps) prefetch(step + 1);

        const int tcol = 16 * w + lr;  // this lane's token inside the step
        const float el_t = bf.ell[tcol];

        // c_t fragments: B operand of (a) and of (d)
        bf16x8 cf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cf[ks] = *reinterpret_cast<const bf16x8 *>(&bf.c[tcol][32 * ks + 8 * lb]);

        // x fragments, token-contracted: slot s < 4 is token 32*pr + 4*lb + s, s >= 4 adds 16
        bf16x8 xf[2][2];
#pragma unroll
        for (int pr = 0; pr < 2; ++pr)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt) {
                const bf16_t *a0 = &bf.x[32 * pr + 4 * lb + (lr >> 2)][16 * pt + 4 * (lr & 3)];
                xf[pr][pt] = cat(lds_read_tr(a0), lds_read_tr(a0 + 16 * kXPitch));
            }

        // (a) + (b): M^T tiles for key blocks jt <= w, packed as B operands of (c)
        bf16x8 mf[2];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            bf16x4 m4 = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
            if (jt <= w) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 bfr = *reinterpret_cast<const bf16x8 *>(&bf.b[16 * jt + lr][32 * ks + 8 * lb]);
                    acc = mfma16(bfr, cf[ks], acc);
                }
                const f32x4 el_j = *reinterpret_cast<const f32x4 *>(&bf.ell[16 * jt + 4 * lb]);
                const f32x4 dt_j = *reinterpret_cast<const f32x4 *>(&bf.dtv[16 * jt + 4 * lb]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int j = 16 * jt + 4 * lb + i;
                    const float val = acc[i] * fast_exp2(el_t - el_j[i]) * dt_j[i];
                    m4[i] = (bf16_t)((j <= tcol) ? val : 0.f);
                }
            }
            if (jt & 1)
                mf[jt >> 1] = cat(__builtin_shufflevector(mf[jt >> 1], mf[jt >> 1], 0, 1, 2, 3), m4);
            else
                mf[jt >> 1] = cat(m4, m4);
        }

        // (c) intra-step part and (d) carried-state part of Y^T[p, t]
        f32x4 yacc[2], yin[2];
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            yacc[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
            yin[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
                if (2 * pr <= w) yacc[pt] = mfma16(xf[pr][pt], mf[pr], yacc[pt]);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 sf = *reinterpret_cast<const bf16x8 *>(&lds.s[cur][16 * pt + lr][32 * ks + 8 * lb]);
                yin[pt] = mfma16(sf, cf[ks], yin[pt]);
            }
        }
        {
            const int t = step * kQ + tcol;
            const float carry = fast_exp2(el_t);
            if (t < T) {
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const int pp = 16 * pt + 4 * lb;
                    bf16x4 out;
                    if (D) {
                        const bf16x4 xv = *reinterpret_cast<const bf16x4 *>(&bf.x[tcol][pp]);
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            out[i] = (bf16_t)(yacc[pt][i] + carry * yin[pt][i] + Dh * (float)xv[i]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) out[i] = (bf16_t)(yacc[pt][i] + carry * yin[pt][i]);
                    }
                    *reinterpret_cast<bf16x4 *>(y + ((size_t)t * H + h) * P + p0 + pp) = out;
                }
            }
        }

        // (e) state update for the rows this wave owns
        {
            const float decay_q = fast_exp2(bf.ell[kQ - 1]);
            f32x4 wj[2][2];
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                wj[pr][0] = *reinterpret_cast<const f32x4 *>(&bf.wv[32 * pr + 4 * lb]);
                wj[pr][1] = *reinterpret_cast<const f32x4 *>(&bf.wv[32 * pr + 16 + 4 * lb]);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] *= decay_q;
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    const bf16_t *a0 = &bf.b[32 * pr + 4 * lb + (lr >> 2)][nbase + 16 * nt + 4 * (lr & 3)];
                    const bf16x4 lo = lds_read_tr(a0), hi = lds_read_tr(a0 + 16 * L::kCP);
                    bf16x8 bw;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        bw[i] = (bf16_t)((float)lo[i] * wj[pr][0][i]);
                        bw[4 + i] = (bf16_t)((float)hi[i] * wj[pr][1][i]);
                    }
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt) sacc[nt][pt] = mfma16(bw, xf[pr][pt], sacc[nt][pt]);
                }
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
        if (step + 1 < nsteps) commit(cur ^ 1);
        __syncthreads();
    }

    if (S_out) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                *reinterpret_cast<f32x4 *>(S_out + ((size_t)h * P + p0 + pt * 16 + lr) * NS + nbase + nt * 16 +
                                           lb * 4) = sacc[nt][pt];
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
    (void)G;
    return io == STRD_BF16 && T >= 1 && (n == 64 || n == 128) && P % kPB == 0 &&
           (long long)H * (P / kPB) < (1 << 24);
}

int ssd_mfma(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
             const float *S_in, void *y, float *S_out, int T, int H, int P, int G, int n, hipStream_t st) {
    if (n == 128) return launch<128>(x, dt, A, B, C, D, S_in, y, S_out, T, H, P, G, st);
    if (n == 64) return launch<64>(x, dt, A, B, C, D, S_in, y, S_out, T, H, P, G, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
