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

// Causal depthwise convolution over the token axis with zero history, then SiLU:
//   o[t, c] = silu(b[c] + sum_{k < W} w[c, k] * in[t - (W - 1) + k, c])
// One thread = 8 adjacent channels of one token; the channel decides the output tensor
// (x | B | C are adjacent column ranges of the input rows).
template <typename T>
__global__ __launch_bounds__(kThreads) void conv1d_silu_kernel(const T *__restrict__ in, int ld, const T *__restrict__ w,
                                                               const T *__restrict__ b, T *__restrict__ xo,
                                                               T *__restrict__ Bo, T *__restrict__ Co, int Tn, int Cx,
                                                               int Cb, int W) {
    typedef typename Vec8<T>::type V;
    const int Ct = Cx + 2 * Cb, vecs = Ct / 8;
    const long long gid = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= (long long)Tn * vecs) return;
    const int t = (int)(gid / vecs), c0 = (int)(gid % vecs) * 8;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = b ? to_f32(b[c0 + e]) : 0.f;
    for (int k = 0; k < W; ++k) {
        const int ts = t - (W - 1) + k;
        if (ts < 0) continue;
        const V v = *reinterpret_cast<const V *>(in + (size_t)ts * ld + c0);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(to_f32(w[(size_t)(c0 + e) * W + k]), to_f32((T)v[e]), acc[e]);
    }
    V o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = from_f32<T>(silu(acc[e]));
    T *dst = c0 < Cx ? xo + (size_t)t * Cx + c0
                     : c0 < Cx + Cb ? Bo + (size_t)t * Cb + (c0 - Cx) : Co + (size_t)t * Cb + (c0 - Cx - Cb);
    *reinterpret_cast<V *>(dst) = o;
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

int glue_rmsnorm(const void *x, const void *w, void *out, int T, int d, float eps, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        rmsnorm_kernel<E><<<T, kThreads, 0, st>>>((const E *)x, (const E *)w, (E *)out, d, eps);
    });
}

int glue_gated_rmsnorm(const void *y, const void *z, int ldz, const void *w, void *out, int T, int D, int groups,
                       float eps, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    return by_dtype(io, [&](auto *tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        gated_rmsnorm_kernel<E><<<T * groups, kThreads, 0, st>>>((const E *)y, (const E *)z, (const E *)w, (E *)out, D, ldz,
                                                               groups, eps);
    });
}

int glue_conv1d_silu(const void *in, int ld, const void *w, const void *b, void *xo, void *Bo, void *Co, int T, int Cx,
                     int Cb, int W, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    const long long n = (long long)T * ((Cx + 2 * Cb) / 8);
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
