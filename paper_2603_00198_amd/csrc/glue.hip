// Block glue of a hybrid layer around the mixers (everything between the projections and the
// scan / attention that is not a matrix product): pre-norm, the short causal convolution with
// SiLU that Mamba-2 applies to x, B, C, the softplus of dt, and the gated RMS norm after the scan.
// The paper takes these from the Mamba-2 block it builds on and does not restate them; they are
// elementwise or row-local, bound by HBM, and computed in fp32 from bf16 or fp32 tensors with one
// rounding on output.
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

__device__ __forceinline__ float silu(float v) { return v / (1.f + __expf(-v)); }

__device__ __forceinline__ float block_sum(float v, float *red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    const int w = threadIdx.x / kWave;
    __syncthreads();  // red may still be read from the previous use
    if ((threadIdx.x & (kWave - 1)) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kThreads / kWave; ++i) t += red[i];  // fixed order
    return t;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// out[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * w.  One workgroup per row.
template <typename T>
__global__ __launch_bounds__(kThreads) void rmsnorm_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                           T *__restrict__ out, int d, float eps) {
    __shared__ float red[kThreads / kWave];
    const T *xr = x + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += kThreads) {
        const float v = to_f32(xr[c]);
        ss = fmaf(v, v, ss);
    }
    const float inv = rsqrtf(block_sum(ss, red) / (float)d + eps);
    T *orow = out + (size_t)blockIdx.x * d;
    for (int c = threadIdx.x; c < d; c += kThreads) orow[c] = from_f32<T>(to_f32(xr[c]) * inv * to_f32(w[c]));
}

// Same, one wave per row with 8-element vectors (d % 8 == 0, 16-byte aligned rows): no barrier,
// the second pass re-reads the row from the cache.
template <typename T>
__global__ __launch_bounds__(kThreads) void rmsnorm_vec_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                               T *__restrict__ out, int Tn, int d, float eps) {
    typedef typename Vec8<T>::type V;
    const int row = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    if (row >= Tn) return;
    const V *xr = reinterpret_cast<const V *>(x + (size_t)row * d);
    const V *wr = reinterpret_cast<const V *>(w);
    V *orow = reinterpret_cast<V *>(out + (size_t)row * d);
    float ss = 0.f;
    for (int c = lane; c < d / 8; c += kWave) {
        const V v = xr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(to_f32((T)v[e]), to_f32((T)v[e]), ss);
    }
    const float inv = rsqrtf(wave_sum(ss) / (float)d + eps);
    for (int c = lane; c < d / 8; c += kWave) {
        const V v = xr[c], wv = wr[c];
        V o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = from_f32<T>(to_f32((T)v[e]) * inv * to_f32((T)wv[e]));
        orow[c] = o;
    }
}

// v = y * silu(z); out = v / sqrt(mean over the group of v^2 + eps) * w.  One workgroup per (row, group).
template <typename T>
__global__ __launch_bounds__(kThreads) void gated_rmsnorm_kernel(const T *__restrict__ y, const T *__restrict__ z,
                                                                 const T *__restrict__ w, T *__restrict__ out, int D,
                                                                 int ldz, int groups, float eps) {
    __shared__ float red[kThreads / kWave];
    const int row = blockIdx.x / groups, g = blockIdx.x % groups, gs = D / groups;
    const T *yr = y + (size_t)row * D + g * gs, *zr = z + (size_t)row * ldz + g * gs;
    float ss = 0.f;
    for (int c = threadIdx.x; c < gs; c += kThreads) {
        const float v = to_f32(yr[c]) * silu(to_f32(zr[c]));
        ss = fmaf(v, v, ss);
    }
    const float inv = rsqrtf(block_sum(ss, red) / (float)gs + eps);
    T *orow = out + (size_t)row * D + g * gs;
    for (int c = threadIdx.x; c < gs; c += kThreads)
        orow[c] = from_f32<T>(to_f32(yr[c]) * silu(to_f32(zr[c])) * inv * to_f32(w[g * gs + c]));
}

// Same, one wave per (row, group) with 8-element vectors; the gated values of up to 4 vectors per
// lane stay in registers between the two passes (groups of up to 2048 channels), longer groups
// recompute them.
template <typename T>
__global__ __launch_bounds__(kThreads) void gated_rmsnorm_vec_kernel(const T *__restrict__ y, const T *__restrict__ z,
                                                                     const T *__restrict__ w, T *__restrict__ out,
                                                                     long long units, int D, int ldz, int groups,
                                                                     float eps) {
    typedef typename Vec8<T>::type V;
    constexpr int kKeep = 4;
    const long long unit = (long long)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    if (unit >= units) return;
    const int row = (int)(unit / groups), g = (int)(unit % groups), gs = D / groups, nv = gs / 8;
    const V *yr = reinterpret_cast<const V *>(y + (size_t)row * D + (size_t)g * gs);
    const V *zr = reinterpret_cast<const V *>(z + (size_t)row * ldz + (size_t)g * gs);
    const V *wr = reinterpret_cast<const V *>(w + (size_t)g * gs);
    V *orow = reinterpret_cast<V *>(out + (size_t)row * D + (size_t)g * gs);
    float keep[kKeep][8];
    float ss = 0.f;
    int i = 0;
    for (int c = lane; c < nv; c += kWave, ++i) {
        const V yv = yr[c], zv = zr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = to_f32((T)yv[e]) * silu(to_f32((T)zv[e]));
            ss = fmaf(v, v, ss);
            if (i < kKeep) keep[i < kKeep ? i : 0][e] = v;
        }
    }
    const float inv = rsqrtf(wave_sum(ss) / (float)gs + eps);
    i = 0;
    for (int c = lane; c < nv; c += kWave, ++i) {
        const V wv = wr[c];
        V o;
        if (i < kKeep) {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = from_f32<T>(keep[i < kKeep ? i : 0][e] * inv * to_f32((T)wv[e]));
        } else {
            const V yv = yr[c], zv = zr[c];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                o[e] = from_f32<T>(to_f32((T)yv[e]) * silu(to_f32((T)zv[e])) * inv * to_f32((T)wv[e]));
        }
        orow[c] = o;
    }
}

// Causal depthwise convolution over the token axis with zero history, then SiLU:
//   o[t, c] = silu(b[c] + sum_{k < W} w[c, k] * in[t - (W - 1) + k, c])
// One thread = 8 adjacent channels of kTok consecutive tokens: it slides a window of W rows down
// its tokens (W <= kMaxW), so each input row is read 1 + (W - 1) / kTok times; lanes run along the
// channels (coalesced rows).  The channel decides the output tensor (x | B | C are adjacent column
// ranges of the input rows).
constexpr int kTok = 8, kMaxW = 4;

template <typename T>
__global__ __launch_bounds__(kThreads) void conv1d_silu_kernel(const T *__restrict__ in, int ld, const T *__restrict__ w,
                                                               const T *__restrict__ b, T *__restrict__ xo,
                                                               T *__restrict__ Bo, T *__restrict__ Co, int Tn, int Cx,
                                                               int Cb, int W) {
    typedef typename Vec8<T>::type V;
    const int Ct = Cx + 2 * Cb, vecs = Ct / 8;
    const long long gid = (long long)blockIdx.x * kThreads + threadIdx.x;
    const int tblocks = (Tn + kTok - 1) / kTok;
    if (gid >= (long long)tblocks * vecs) return;
    const int t0 = (int)(gid / vecs) * kTok, c0 = (int)(gid % vecs) * 8;
    // rows t0 - (kMaxW - 1) .. t0 + kTok - 1, all requested before any arithmetic (rows outside the
    // sequence: a valid row is read and replaced by zeros / not stored)
    V rows[kTok + kMaxW - 1];
#pragma unroll
    for (int j = 0; j < kTok + kMaxW - 1; ++j) {
        const int ts = min(max(t0 - (kMaxW - 1) + j, 0), Tn - 1);
        rows[j] = *reinterpret_cast<const V *>(in + (size_t)ts * ld + c0);
    }
    float wt[8][kMaxW], bias[8];  // tap k of a width-W filter reads row t - (W - 1) + k: window slot k + kMaxW - W
    if (b) {
        const V bv = *reinterpret_cast<const V *>(b + c0);
#pragma unroll
        for (int e = 0; e < 8; ++e) bias[e] = to_f32((T)bv[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) bias[e] = 0.f;
    }
    if (W == kMaxW) {  // uniform: the 8 channels' taps are 32 adjacent weights
        V wv[kMaxW];
#pragma unroll
        for (int j = 0; j < kMaxW; ++j) wv[j] = *reinterpret_cast<const V *>(w + (size_t)c0 * kMaxW + 8 * j);
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int j = 0; j < kMaxW; ++j) wt[e][j] = to_f32((T)wv[(e * kMaxW + j) / 8][(e * kMaxW + j) % 8]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int j = 0; j < kMaxW; ++j) {
                const int k = j - (kMaxW - W);
                wt[e][j] = k >= 0 ? to_f32(w[(size_t)(c0 + e) * W + k]) : 0.f;
            }
    }
    T *dst = c0 < Cx ? xo + c0 : c0 < Cx + Cb ? Bo + (c0 - Cx) : Co + (c0 - Cx - Cb);
    const int pitch = c0 < Cx ? Cx : Cb;
#pragma unroll
    for (int i = 0; i < kTok; ++i) {
        const int t = t0 + i;
        if (t < Tn) {
            V o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float acc = bias[e];
#pragma unroll
                for (int j = 0; j < kMaxW; ++j) {
                    const float v = (t - (kMaxW - 1) + j >= 0) ? to_f32((T)rows[i + j][e]) : 0.f;  // zero history
                    acc = fmaf(wt[e][j], v, acc);
                }
                o[e] = from_f32<T>(silu(acc));
            }
            *reinterpret_cast<V *>(dst + (size_t)t * pitch) = o;
        }
    }
}

// dt[t, h] = softplus(raw[t, col0 + h] + bias[h]) = log(1 + exp(.)), fp32 out
template <typename T>
__global__ __launch_bounds__(kThreads) void softplus_dt_kernel(const T *__restrict__ raw, int ld, int col0,
                                                               const float *__restrict__ bias, float *__restrict__ dt,
                                                               int Tn, int H) {
    const long long gid = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= (long long)Tn * H) return;
    const int t = (int)(gid / H), h = (int)(gid % H);
    const float v = to_f32(raw[(size_t)t * ld + col0 + h]) + (bias ? bias[h] : 0.f);
    dt[gid] = v > 20.f ? v : log1pf(__expf(v));
}

template <typename F> int by_dtype(strd_dtype io, F &&f) {
    if (io == STRD_F32) f((float *)nullptr); else f((bf16_t *)nullptr);
    return launch_status();
}

}  // namespace

int glue_conv_max_width() { return kMaxW; }

int glue_rmsnorm(const void *x, const void *w, void *out, int T, int d, float eps, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    const size_t es = io == STRD_F32 ? 4 : 2;
    const bool vec = d % 8 == 0 && !((uintptr_t)x % (8 * es)) && !((uintptr_t)w % (8 * es)) && !((uintptr_t)out % (8 * es));
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (vec)
            rmsnorm_vec_kernel<E><<<ceil_div(T, kThreads / kWave), kThreads, 0, st>>>((const E *)x, (const E *)w, (E *)out, T,
                                                                                    d, eps);
        else
            rmsnorm_kernel<E><<<T, kThreads, 0, st>>>((const E *)x, (const E *)w, (E *)out, d, eps);
    });
}

int glue_gated_rmsnorm(const void *y, const void *z, int ldz, const void *w, void *out, int T, int D, int groups,
                       float eps, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    const size_t es = io == STRD_F32 ? 4 : 2;
    const bool vec = (D / groups) % 8 == 0 && ldz % 8 == 0 && !((uintptr_t)y % (8 * es)) && !((uintptr_t)z % (8 * es)) &&
                     !((uintptr_t)w % (8 * es)) && !((uintptr_t)out % (8 * es));
    const long long units = (long long)T * groups;
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (vec)
            gated_rmsnorm_vec_kernel<E><<<(int)((units + kThreads / kWave - 1) / (kThreads / kWave)), kThreads, 0, st>>>(
                (const E *)y, (const E *)z, (const E *)w, (E *)out, units, D, ldz, groups, eps);
        else
            gated_rmsnorm_kernel<E><<<T * groups, kThreads, 0, st>>>((const E *)y, (const E *)z, (const E *)w, (E *)out, D,
                                                                   ldz, groups, eps);
    });
}

int glue_conv1d_silu(const void *in, int ld, const void *w, const void *b, void *xo, void *Bo, void *Co, int T, int Cx,
                     int Cb, int W, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    const long long n = (long long)ceil_div(T, kTok) * ((Cx + 2 * Cb) / 8);
    const int grid = (int)((n + kThreads - 1) / kThreads);
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        conv1d_silu_kernel<E><<<grid, kThreads, 0, st>>>((const E *)in, ld, (const E *)w, (const E *)b, (E *)xo, (E *)Bo,
                                                        (E *)Co, T, Cx, Cb, W);
    });
}

int glue_softplus_dt(const void *raw, int ld, int col0, const float *bias, float *dt, int T, int H, strd_dtype io,
                     hipStream_t st) {
    if (T == 0) return STRD_OK;
    const long long n = (long long)T * H;
    const int grid = (int)((n + kThreads - 1) / kThreads);
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        softplus_dt_kernel<E><<<grid, kThreads, 0, st>>>((const E *)raw, ld, col0, bias, dt, T, H);
    });
}

}  // namespace strd
