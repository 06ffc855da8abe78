// attn_prefill on bf16 matrix cores: causal softmax attention with grouped-query heads (paper
// App. "Attention via Kernel Functions", first equation), flash-style: the score matrix is
// produced and consumed tile by tile with a running max and sum per query.
//
// One workgroup = 4 waves = one query head x 128 consecutive query positions; wave w owns 32 of
// them.  Tiles are computed transposed (v_mfma_f32_32x32x16_bf16):
//     S^T[key, t] = K_tile . Q^T        A = key rows from LDS, B = query fragments in registers
//     O^T[d,  t] += V_tile^T . P^T      A = V read with the transposing LDS load, B = P^T
// so a lane owns one query column: its running max, running sum and the rescale factor are
// per-lane scalars, and the fp32 score accumulators of a 32-key tile, converted to bf16, are
// already laid out as the B operand of the second product (8 consecutive accumulator registers
// = the 8 contraction slots of a lane; V is read with the matching key permutation).
// K and V stream through LDS in 64-key chunks, double-buffered, shared by the 4 waves; the
// next chunk is prefetched into registers during the current one.  Workgroups are issued
// longest-first (last query block first), heads of one kv group adjacent.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBM = 128;  // query positions per workgroup
constexpr int kKC = 64;   // keys per LDS chunk
constexpr float kLog2e = 1.4426950408889634f;

template <int D>
struct Tile {
    static constexpr int kPitch = D + 8;
    bf16_t k[2][kKC][kPitch];
    bf16_t v[2][kKC][kPitch];
};

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Transposing LDS read: within 16 lanes, lane r passes &tile[k0 + r/4][c0 + 4*(r%4)] and
// receives tile[k0..k0+3][c0 + r].
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t *p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p));
    return __builtin_bit_cast(bf16x4, v);
}
__device__ __forceinline__ bf16x8 cat(bf16x4 lo, bf16x4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                             const bf16_t *__restrict__ v, bf16_t *__restrict__ o, int T,
                                                             int Hq, int Hkv, float scale2, int nqb) {
    constexpr int KS = D / 16, DT = D / 32, VR = D / 8, VPT = kKC * VR / kThreads;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    Tile<D> &lds = *reinterpret_cast<Tile<D> *>(smem_raw);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lc = lane & 31, half = lane >> 5;
    const int h = blockIdx.x % Hq, qb = nqb - 1 - blockIdx.x / Hq, kvh = h / (Hq / Hkv);
    const int t0 = qb * kBM;
    const int tq = t0 + 32 * w + lc;             // this lane's query position
    const int wq0 = t0 + 32 * w;                 // first query of the wave
    const int wmax = min(T - 1, wq0 + 31);       // last key any query of the wave may see
    const int nkeys = min(T, t0 + kBM);
    const int nchunk = (nkeys + kKC - 1) / kKC;

    bf16x8 bq[KS];
    {
        const bf16_t *qp = q + ((size_t)min(tq, T - 1) * Hq + h) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bq[ks] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ks + 8 * half);
    }

    uint4 sk[VPT], sv[VPT];
    auto stage_load = [&](int chunk) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int e = tid + i * kThreads, r = e / VR, cv = e % VR;
            const size_t off = ((size_t)min(chunk * kKC + r, T - 1) * Hkv + kvh) * D + cv * 8;
            sk[i] = *reinterpret_cast<const uint4 *>(k + off);
            sv[i] = *reinterpret_cast<const uint4 *>(v + off);
        }
    };
    auto stage_store = [&](int b) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int e = tid + i * kThreads, r = e / VR, cv = e % VR;
            *reinterpret_cast<uint4 *>(&lds.k[b][r][cv * 8]) = sk[i];
            *reinterpret_cast<uint4 *>(&lds.v[b][r][cv * 8]) = sv[i];
        }
    };

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane half's share of the row sum

    // lane-dependent parts of the transposed V read
    const int vb = lane >> 4, vr = lane & 15;
    const int v_krow = 4 * (vb >> 1) + (vr >> 2), v_col = 16 * (vb & 1) + 4 * (vr & 3);

    stage_load(0);
    stage_store(0);
    __syncthreads();
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int cur = chunk & 1;
        stage_load(min(chunk + 1, nchunk - 1));
#pragma unroll
        for (int kt = 0; kt < kKC / 32; ++kt) {
            const int kb = chunk * kKC + 32 * kt;
            if (kb <= wmax) {  // uniform per wave
                f32x16 sacc;
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&lds.k[cur][32 * kt + lc][16 * ks + 8 * half]);
                    sacc = mfma32(a, bq[ks], sacc);
                }
                const bool diag = kb + 31 > wq0;  // some (key, query) pair of the tile is masked
                float z[16], tm = -INFINITY;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    z[i] = sacc[i] * scale2;
                    if (diag && kb + 8 * (i / 4) + 4 * half + (i % 4) > tq) z[i] = -INFINITY;
                    tm = fmaxf(tm, z[i]);
                }
                tm = fmaxf(tm, __shfl_xor(tm, 32, kWave));
                const float nm = fmaxf(m_run, tm);  // finite: key 0 is visible to every query
                if (__any(nm > m_run)) {
                    const float corr = ex2(m_run - nm);
                    l_run *= corr;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[dt][i] *= corr;
                    m_run = nm;
                }
                float ps = 0.f;
                bf16x8 pf[2];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = ex2(z[i] - m_run);
                    ps += p;
                    pf[i >> 3][i & 7] = (bf16_t)p;
                }
                l_run += ps;
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) {
                    const bf16_t *vp = &lds.v[cur][32 * kt + 16 * ks2 + v_krow][v_col];
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const bf16x8 vf = cat(lds_read_tr(vp + 32 * dt), lds_read_tr(vp + 32 * dt + 8 * Tile<D>::kPitch));
                        oacc[dt] = mfma32(vf, pf[ks2], oacc[dt]);
                    }
                }
            }
        }
        stage_store(cur ^ 1);
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (tq < T) {
        const float inv = 1.f / l_tot;
        bf16_t *op = o + ((size_t)tq * Hq + h) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = (bf16_t)(oacc[dt][4 * i4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + 32 * dt + 8 * i4 + 4 * half) = out;
            }
    }
}

template <int D>
int launch(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, float scale, hipStream_t st) {
    const size_t smem = sizeof(Tile<D>);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma_kernel<D>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return STRD_EHIP;
        configured = true;
    }
    const int nqb = ceil_div(T, kBM);
    attn_mfma_kernel<D><<<nqb * Hq, kThreads, smem, st>>>((const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                                                          (bf16_t *)o, T, Hq, Hkv, scale * kLog2e, nqb);
    return launch_status();
}

}  // namespace

bool attn_mfma_supported(int T, int Hq, int Hkv, int d, strd_dtype io) {
    (void)Hkv;
    return io == STRD_BF16 && T >= 1 && (d == 64 || d == 128) && (long long)ceil_div(T, kBM) * Hq < (1LL << 30);
}

int attn_mfma(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d, float scale,
              hipStream_t st) {
    if (d == 128) return launch<128>(q, k, v, o, T, Hq, Hkv, scale, st);
    if (d == 64) return launch<64>(q, k, v, o, T, Hq, Hkv, scale, st);
    return STRD_EUNSUPPORTED;
}

}  // namespace strd
