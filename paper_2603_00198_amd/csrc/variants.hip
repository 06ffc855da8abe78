// Variants around the reduced prefill:
//  * avgpool: the average-pooling reduction that the paper's "Reduction Types" ablation sets
//    against query-based selection.  The N vision rows are cut into K consecutive windows
//    [floor(jN/K), floor((j+1)N/K)), each replaced by its mean; the text rows follow unchanged.
//    Bandwidth kernel: one read of N+M rows, one write of K+M rows.
//  * ssd_decode_step / attn_decode_step: the hand-off of what a reduced prefill leaves behind --
//    the recurrent state S (paper Eq. ssm_state_update / ssm_output with one token) and the
//    key/value rows of the K+M survivors -- to single-token generation.  Both are bound by HBM:
//    the state is read and written once, the cache is read once.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 256;

template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    typedef __bf16 type __attribute__((ext_vector_type(8)));
};
template <> struct Vec8<float> {
    typedef float type __attribute__((ext_vector_type(8)));
};

__host__ __device__ __forceinline__ int window_edge(int j, int N, int K) { return (int)(((long long)j * N) / K); }

// ------------------------------------------------------------------ avgpool ---------------
// One thread per 8-channel vector of an output row; the rows of its window are read four at a time.
template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_vec_kernel(const T *__restrict__ src, T *__restrict__ dst, int N,
                                                               int K, int rows_out, int vpr) {
    typedef typename Vec8<T>::type V;
    const long long e = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (e >= (long long)rows_out * vpr) return;
    const int r = (int)(e / vpr), c = (int)(e - (long long)r * vpr);
    const V *s = reinterpret_cast<const V *>(src) + c;
    V *d = reinterpret_cast<V *>(dst) + (size_t)r * vpr + c;
    if (r >= K) {  // text row
        *d = s[(size_t)(N + (r - K)) * vpr];
        return;
    }
    const int lo = window_edge(r, N, K), hi = window_edge(r + 1, N, K);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r0 = lo; r0 < hi; r0 += 4) {
        V v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (r0 + u < hi) v[u] = __builtin_nontemporal_load(s + (size_t)(r0 + u) * vpr);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (r0 + u < hi) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += to_f32((T)v[u][i]);
            }
    }
    const float cnt = (float)(hi - lo);
    V o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = from_f32<T>(acc[i] / cnt);
    *d = o;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_kernel(const T *__restrict__ src, T *__restrict__ dst, int N, int K,
                                                           int rows_out, int D) {
    const long long e = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (e >= (long long)rows_out * D) return;
    const int r = (int)(e / D), c = (int)(e - (long long)r * D);
    if (r >= K) {
        dst[e] = src[(size_t)(N + (r - K)) * D + c];
        return;
    }
    const int lo = window_edge(r, N, K), hi = window_edge(r + 1, N, K);
    float acc = 0.f;
    for (int q = lo; q < hi; ++q) acc += to_f32(src[(size_t)q * D + c]);
    dst[e] = from_f32<T>(acc / (float)(hi - lo));
}

// A pooled token takes the position of the first row of its window.
__global__ __launch_bounds__(kThreads) void avgpool_pos_kernel(const int32_t *__restrict__ pos_in,
                                                               int32_t *__restrict__ pos_out, int N, int K,
                                                               int rows_out) {
    const int r = blockIdx.x * kThreads + threadIdx.x;
    if (r >= rows_out) return;
    const int sr = r < K ? window_edge(r, N, K) : N + (r - K);
    pos_out[r] = pos_in ? pos_in[sr] : sr;
}

template <typename T>
int avgpool_typed(const void *src, void *dst, int N, int M, int K, int D, hipStream_t st) {
    const int rows_out = K + M;
    const bool vec = D % 8 == 0 && (uintptr_t)src % (8 * sizeof(T)) == 0 && (uintptr_t)dst % (8 * sizeof(T)) == 0;
    const long long work = (long long)rows_out * (vec ? D / 8 : D);
    const long long blocks = (work + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    if (blocks == 0) return STRD_OK;
    if (vec)
        avgpool_vec_kernel<T><<<(unsigned)blocks, kThreads, 0, st>>>((const T *)src, (T *)dst, N, K, rows_out, D / 8);
    else
        avgpool_kernel<T><<<(unsigned)blocks, kThreads, 0, st>>>((const T *)src, (T *)dst, N, K, rows_out, D);
    return launch_status();
}

// ------------------------------------------------------------------ ssd_decode_step -------
// S'[h,p,:] = exp(dt_h A_h) S[h,p,:] + dt_h x[h,p] b_g(h);  y[h,p] = S'[h,p,:] . c_g(h) + D_h x[h,p].
// L lanes share one (h, p) row of the state, VW state columns per lane and trip; the dot
// product is finished by a butterfly over the L lanes.
template <typename T, int L, int VW>
__global__ __launch_bounds__(kThreads) void ssd_decode_kernel(const T *__restrict__ x, const float *__restrict__ dt,
                                                              const float *__restrict__ A, const T *__restrict__ B,
                                                              const T *__restrict__ C, const float *__restrict__ D,
                                                              float *__restrict__ S, T *__restrict__ y, int H, int P,
                                                              int G, int n) {
    const int row = (blockIdx.x * kThreads + threadIdx.x) / L;  // h * P + p
    const int sub = threadIdx.x % L;
    const bool live = row < H * P;
    const int rr = live ? row : 0;
    const int h = rr / P, g = h / (H / G);
    const float dth = dt[h], decay = __expf(dth * A[h]);
    const float xv = to_f32(x[rr]);
    const float dx = dth * xv;
    float *Sr = S + (size_t)rr * n;
    const T *b = B + (size_t)g * n, *c = C + (size_t)g * n;
    float acc = 0.f;
    if (live) {
        for (int q = sub * VW; q < n; q += L * VW) {
            if (VW == 4) {
                float4 sv = *reinterpret_cast<const float4 *>(Sr + q);
                sv.x = fmaf(decay, sv.x, dx * to_f32(b[q + 0]));
                sv.y = fmaf(decay, sv.y, dx * to_f32(b[q + 1]));
                sv.z = fmaf(decay, sv.z, dx * to_f32(b[q + 2]));
                sv.w = fmaf(decay, sv.w, dx * to_f32(b[q + 3]));
                *reinterpret_cast<float4 *>(Sr + q) = sv;
                acc = fmaf(sv.x, to_f32(c[q + 0]), acc);
                acc = fmaf(sv.y, to_f32(c[q + 1]), acc);
                acc = fmaf(sv.z, to_f32(c[q + 2]), acc);
                acc = fmaf(sv.w, to_f32(c[q + 3]), acc);
            } else {
                const float sv = fmaf(decay, Sr[q], dx * to_f32(b[q]));
                Sr[q] = sv;
                acc = fmaf(sv, to_f32(c[q]), acc);
            }
        }
    }
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
    if (live && sub == 0) y[rr] = from_f32<T>(acc + (D ? D[h] * xv : 0.f));
}

template <typename T>
int ssd_decode_typed(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
                     float *S, void *y, int H, int P, int G, int n, hipStream_t st) {
    const long long rows = (long long)H * P;
#define STRD_DECODE(LL, VV)                                                                                         \
    ssd_decode_kernel<T, LL, VV><<<(unsigned)((rows * LL + kThreads - 1) / kThreads), kThreads, 0, st>>>(            \
        (const T *)x, dt, A, (const T *)B, (const T *)C, D, S, (T *)y, H, P, G, n)
    const bool v4 = n % 4 == 0 && (uintptr_t)S % 16 == 0;
    if (v4 && n >= 128) STRD_DECODE(32, 4);
    else if (v4 && n >= 64) STRD_DECODE(16, 4);
    else if (v4) STRD_DECODE(4, 4);
    else STRD_DECODE(16, 1);
#undef STRD_DECODE
    return launch_status();
}

// ------------------------------------------------------------------ attn_decode_step ------
// o^h = sum_j softmax_j(scale q^h . k_j) v_j over all T cached rows, for one new query per head.
// Pass 1: workgroup (split s, kv head) = 4 waves, each walking a quarter of the split's tokens;
// LPT = d / 8 lanes share a token (8 channels each); a wave takes 16 tokens per trip and loads the
// next trip while it folds the current one; the split length is chosen so that the whole grid is
// about one resident round of the chip.  Every lane group keeps
// its own running (max, sum, accumulator) for the REP query heads of the kv head; the groups of a
// wave are merged by shuffles, the 4 waves through LDS, and the workgroup writes one partial
// (max, sum, accumulator) per query head.  Pass 2 merges the partials of all splits, 32 channels
// of one head per workgroup.  Scores are kept in log2 units.
constexpr float kNegBig = -1.0e30f;  // stands for "no key seen yet": finite, so differences stay finite
constexpr int kDecWaves = 4;
constexpr int kTokSplit = 64;    // slice granularity: one 16-token trip per wave
constexpr int kMaxSplits = 1024;

template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
#define STRD_DPP_ADD(ctrl) \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, true))
    STRD_DPP_ADD(0xB1);   // quad_perm [1,0,3,2]
    STRD_DPP_ADD(0x4E);   // quad_perm [2,3,0,1]
    STRD_DPP_ADD(0x141);  // row_half_mirror
    if (LPT == 16) STRD_DPP_ADD(0x140);  // row_mirror
#undef STRD_DPP_ADD
    return v;
}

template <typename T, int LPT, int REP>
__global__ __launch_bounds__(kDecWaves * kWave) void attn_decode_partial_kernel(
    const T *__restrict__ q, const T *__restrict__ kc, const T *__restrict__ vc, float *__restrict__ part,
    float *__restrict__ ml, int Tn, int Hq, int Hkv, int tok_per_split, float scale_log2) {
    typedef typename Vec8<T>::type V;
    constexpr int d = LPT * 8, TPI = kWave / LPT;
    __shared__ float sm_acc[kDecWaves][REP][d];
    __shared__ float sm_ml[kDecWaves][REP][2];
    const int split = blockIdx.y, hk = blockIdx.x;  // the kv heads of a token range run side by side: whole rows are in flight together
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, sub = lane % LPT, grp = lane / LPT;
    float qv[REP][8], m[REP], l[REP], acc[REP][8];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        const V t = *reinterpret_cast<const V *>(q + (size_t)(hk * REP + r) * d + sub * 8);
        m[r] = kNegBig;
        l[r] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            qv[r][i] = to_f32((T)t[i]) * scale_log2;
            acc[r][i] = 0.f;
        }
    }
    const int per_wave = tok_per_split / kDecWaves;
    const int t_begin = split * tok_per_split + wave * per_wave, t_end = min(Tn, t_begin + per_wave);
    const size_t row_stride = (size_t)Hkv * d;
    const T *kbase = kc + (size_t)hk * d + sub * 8, *vbase = vc + (size_t)hk * d + sub * 8;
    constexpr int kUnroll = 16 / TPI;  // 16 tokens per trip
    // Rows past the end of the cache are clamped to its last row and masked, so every load is
    // unconditional and the next trip's loads are in flight while this trip is computed.
    auto load_trip = [&](int t0, V (&kv)[kUnroll], V (&vv)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = min(t0 + u * TPI + grp, Tn - 1);
            kv[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(kbase + (size_t)t * row_stride));
            vv[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(vbase + (size_t)t * row_stride));
        }
    };
    auto fold_trip = [&](int t0, const V (&kv)[kUnroll], const V (&vv)[kUnroll]) {
        float sc[kUnroll][REP];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool valid = t0 + u * TPI + grp < t_end;
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) dot = fmaf(qv[r][i], to_f32((T)kv[u][i]), dot);
                sc[u][r] = valid ? group_sum<LPT>(dot) : kNegBig;
            }
        }
        // one rescale per trip: the running maximum moves to the maximum over the trip's tokens
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            float mn = m[r];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) mn = fmaxf(mn, sc[u][r]);
            const float corr = exp2f(m[r] - mn);
            m[r] = mn;
            l[r] *= corr;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[r][i] *= corr;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool valid = t0 + u * TPI + grp < t_end;
            float vf[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) vf[i] = to_f32((T)vv[u][i]);
#pragma unroll
            for (int r = 0; r < REP; ++r) {
                const float p = valid ? exp2f(sc[u][r] - m[r]) : 0.f;
                l[r] += p;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[r][i] = fmaf(p, vf[i], acc[r][i]);
            }
        }
    };
    V ka[kUnroll], va[kUnroll], kb[kUnroll], vb[kUnroll];
    load_trip(t_begin < Tn ? t_begin : 0, ka, va);
    for (int t0 = t_begin; t0 < t_end; t0 += 32) {
        load_trip(t0 + 16, kb, vb);
        fold_trip(t0, ka, va);
        load_trip(t0 + 32, ka, va);
        if (t0 + 16 < t_end) fold_trip(t0 + 16, kb, vb);
    }
    // merge the lane groups of the wave
#pragma unroll
    for (int o = LPT; o < kWave; o <<= 1) {
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            const float mo = __shfl_xor(m[r], o, kWave), lo = __shfl_xor(l[r], o, kWave);
            const float mn = fmaxf(m[r], mo);
            const float ca = exp2f(m[r] - mn), cb = exp2f(mo - mn);
            l[r] = l[r] * ca + lo * cb;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[r][i] = acc[r][i] * ca + __shfl_xor(acc[r][i], o, kWave) * cb;
            m[r] = mn;
        }
    }
    if (grp == 0) {
#pragma unroll
        for (int r = 0; r < REP; ++r) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sm_acc[wave][r][sub * 8 + i] = acc[r][i];
            if (sub == 0) {
                sm_ml[wave][r][0] = m[r];
                sm_ml[wave][r][1] = l[r];
            }
        }
    }
    __syncthreads();
    // merge the waves: one thread per (query head, channel)
    for (int e = threadIdx.x; e < REP * d; e += kDecWaves * kWave) {
        const int r = e / d, c = e - r * d;
        float mx = sm_ml[0][r][0];
#pragma unroll
        for (int w = 1; w < kDecWaves; ++w) mx = fmaxf(mx, sm_ml[w][r][0]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float cw = exp2f(sm_ml[w][r][0] - mx);
            num = fmaf(cw, sm_acc[w][r][c], num);
            den = fmaf(cw, sm_ml[w][r][1], den);
        }
        const size_t ph = (size_t)split * Hq + hk * REP + r;
        part[ph * d + c] = num;
        if (c == 0) {
            ml[ph * 2] = mx;
            ml[ph * 2 + 1] = den;
        }
    }
}

// grid (Hq, d / 32), 256 threads: lane c4 = tid % 8 owns 4 channels, the 32 lane groups share the splits.
template <typename T>
__global__ __launch_bounds__(256) void attn_decode_combine_kernel(const float *__restrict__ part,
                                                                  const float *__restrict__ ml, T *__restrict__ o,
                                                                  int nsplit, int Hq, int d) {
    __shared__ float wts[kMaxSplits];
    __shared__ float red[8];
    __shared__ float4 sums[32][8];
    const int h = blockIdx.x, c0 = blockIdx.y * 32, tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    float mloc = kNegBig;
    for (int s = tid; s < nsplit; s += 256) mloc = fmaxf(mloc, ml[((size_t)s * Hq + h) * 2]);
#pragma unroll
    for (int x = 32; x > 0; x >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, x, kWave));
    if (lane == 0) red[wave] = mloc;
    __syncthreads();
    const float mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float dloc = 0.f;
    for (int s = tid; s < nsplit; s += 256) {
        const size_t ph = (size_t)s * Hq + h;
        const float w = exp2f(ml[ph * 2] - mx);
        wts[s] = w;
        dloc = fmaf(w, ml[ph * 2 + 1], dloc);
    }
#pragma unroll
    for (int x = 32; x > 0; x >>= 1) dloc += __shfl_xor(dloc, x, kWave);
    if (lane == 0) red[4 + wave] = dloc;
    __syncthreads();
    const float den = (red[4] + red[5]) + (red[6] + red[7]);
    const int c4 = tid % 8, sg = tid / 8;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *pc = part + (size_t)h * d + c0 + c4 * 4;
    for (int s0 = sg; s0 < nsplit; s0 += 32 * 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = min(s0 + 32 * u, nsplit - 1);
            v[u] = *reinterpret_cast<const float4 *>(pc + (size_t)s * Hq * d);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = s0 + 32 * u < nsplit ? wts[s0 + 32 * u] : 0.f;
            acc.x = fmaf(w, v[u].x, acc.x);
            acc.y = fmaf(w, v[u].y, acc.y);
            acc.z = fmaf(w, v[u].z, acc.z);
            acc.w = fmaf(w, v[u].w, acc.w);
        }
    }
    sums[sg][c4] = acc;
    __syncthreads();
    if (tid < 32) {
        const float *sf = reinterpret_cast<const float *>(&sums[0][0]);
        float num = 0.f;
#pragma unroll
        for (int g = 0; g < 32; ++g) num += sf[g * 32 + tid];  // fixed order
        o[(size_t)h * d + c0 + tid] = from_f32<T>(num / den);
    }
}

// About kDecGroups workgroups in all: one resident round of the chip, several trips per wave.
constexpr int kDecGroups = 700;
inline int decode_tok_per_split(int T, int Hkv) {
    const int want = min(kMaxSplits, max(1, kDecGroups / Hkv));
    return kTokSplit * max(1, ceil_div(T, kTokSplit * want));
}

template <typename T, int LPT>
int attn_decode_typed(const void *q, const void *kc, const void *vc, void *o, int Tn, int Hq, int Hkv, float scale,
                      float *ws, hipStream_t st) {
    const int d = LPT * 8, rep = Hq / Hkv;
    const int tps = decode_tok_per_split(Tn, Hkv), nsplit = ceil_div(Tn, tps);
    float *part = ws, *ml = ws + (size_t)nsplit * Hq * d;
    const float sl2 = scale * 1.4426950408889634f;
    const dim3 grid(Hkv, nsplit);
#define STRD_ADEC(R)                                                                                       \
    attn_decode_partial_kernel<T, LPT, R><<<grid, kDecWaves * kWave, 0, st>>>((const T *)q, (const T *)kc,    \
                                                                              (const T *)vc, part, ml, Tn, Hq, \
                                                                              Hkv, tps, sl2)
    switch (rep) {
    case 1: STRD_ADEC(1); break;
    case 2: STRD_ADEC(2); break;
    case 4: STRD_ADEC(4); break;
    case 8: STRD_ADEC(8); break;
    default: return STRD_EUNSUPPORTED;
    }
#undef STRD_ADEC
    if (hipGetLastError() != hipSuccess) return STRD_EHIP;
    attn_decode_combine_kernel<T><<<dim3(Hq, d / 32), 256, 0, st>>>(part, ml, (T *)o, nsplit, Hq, d);
    return launch_status();
}

}  // namespace

int avgpool_launch(const void *src, void *dst, int N, int M, int K, int D, strd_dtype io, const int32_t *pos_in,
                   int32_t *pos_out, hipStream_t st) {
    const int rows_out = K + M;
    if (rows_out == 0) return STRD_OK;
    int rc = STRD_OK;
    if (src && D > 0)
        rc = io == STRD_BF16 ? avgpool_typed<bf16_t>(src, dst, N, M, K, D, st) : avgpool_typed<float>(src, dst, N, M, K, D, st);
    if (rc != STRD_OK) return rc;
    if (pos_out) {
        avgpool_pos_kernel<<<ceil_div(rows_out, kThreads), kThreads, 0, st>>>(pos_in, pos_out, N, K, rows_out);
        rc = launch_status();
    }
    return rc;
}

int ssd_decode_launch(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
                      float *S, void *y, int H, int P, int G, int n, strd_dtype io, hipStream_t st) {
    return io == STRD_BF16 ? ssd_decode_typed<bf16_t>(x, dt, A, B, C, D, S, y, H, P, G, n, st)
                           : ssd_decode_typed<float>(x, dt, A, B, C, D, S, y, H, P, G, n, st);
}

bool attn_decode_supported(int Hq, int Hkv, int d) {
    const int rep = Hq / Hkv;
    return (d == 64 || d == 128) && (rep == 1 || rep == 2 || rep == 4 || rep == 8);
}

size_t attn_decode_workspace(int T, int Hq, int Hkv, int d) {
    if (T <= 0) return 0;
    const size_t nsplit = (size_t)ceil_div(T, decode_tok_per_split(T, Hkv));
    return nsplit * Hq * (d + 2) * sizeof(float);
}

int attn_decode_launch(const void *q, const void *kc, const void *vc, void *o, int T, int Hq, int Hkv, int d,
                       float scale, strd_dtype io, float *ws, hipStream_t st) {
    if (io == STRD_BF16)
        return d == 128 ? attn_decode_typed<bf16_t, 16>(q, kc, vc, o, T, Hq, Hkv, scale, ws, st)
                        : attn_decode_typed<bf16_t, 8>(q, kc, vc, o, T, Hq, Hkv, scale, ws, st);
    return d == 128 ? attn_decode_typed<float, 16>(q, kc, vc, o, T, Hq, Hkv, scale, ws, st)
                    : attn_decode_typed<float, 8>(q, kc, vc, o, T, Hq, Hkv, scale, ws, st);
}

}  // namespace strd
