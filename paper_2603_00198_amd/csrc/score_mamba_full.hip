// score_mamba_full: the Full Mamba Dynamic importance score (|w_{t,j}| of paper Eq. "ssm_weight", Sec. "Why the Full Mamba Dynamic Fails",
// the variant the decay-free score of Eq. "ssm_importance" is ablated against):
//     s_i = 1/(M*H) * sum_{m,h} dt_i^h * |b_i^{g(h)} . c_m^{g(h)}| * prod_{u=i+1}^{N+m} exp(dt_u^h A^h)
// The decay from vision token i to text row m factors at the vision / text boundary:
//     prod = exp(A^h R_i^h) * exp(A^h T_m^h),  R_i^h = sum_{u=i+1}^{N-1} dt_u^h,  T_m^h = sum_{u=N}^{N+m} dt_u^h
// so u_i^h = dt_i^h exp(A^h R_i^h) <= dt_i^h and v_m^h = exp(A^h T_m^h) <= 1 are made first (a
// blocked suffix sum over the vision tokens and a prefix sum over the text rows; suffix sums
// counted from the boundary are exact to fp32 rounding where the decay is not negligible), then
//     s_i = 1/(M*H) * sum_g sum_m |b_i^g . c_m^g| * sum_{h in g} u_i^h v_m^h.
// This file: the prep kernels and the plain SIMT evaluation (any shape, fp32 or bf16 inputs);
// the matrix-core evaluation lives with the decay-free score kernel it extends.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 64;   // vision tokens per block of the suffix sum

// blockIdx.x < nblk: bs[blk][h] = sum of dt over the block's tokens.  blockIdx.x == nblk: the
// text rows, v_m^h = exp(A^h * sum_{u=N}^{N+m} dt_u^h).  Thread = head (coalesced rows).
__global__ __launch_bounds__(kThreads) void full_prep_sums_kernel(const float *__restrict__ dt,
                                                                  const float *__restrict__ A,
                                                                  float *__restrict__ bs, float *__restrict__ V, int M,
                                                                  int N, int H, int nblk) {
    const int h = blockIdx.y * kThreads + threadIdx.x;
    if (h >= H) return;
    const int blk = blockIdx.x;
    if (blk == nblk) {
        const float a = A[h];
        float run = 0.f;
        for (int m = 0; m < M; ++m) {
            run += dt[(size_t)(N + m) * H + h];
            V[(size_t)m * H + h] = __expf(a * run);
        }
        return;
    }
    const int i0 = blk * kRows, i1 = min(N, i0 + kRows);
    float sum = 0.f;
    for (int i = i0; i < i1; ++i) sum += dt[(size_t)i * H + h];
    bs[(size_t)blk * H + h] = sum;
}

// bs[blk][h] <- sum of dt over all later blocks (exclusive suffix sum, from the boundary outwards)
__global__ __launch_bounds__(kThreads) void full_prep_scan_kernel(float *__restrict__ bs, int H, int nblk) {
    const int h = blockIdx.x * kThreads + threadIdx.x;
    if (h >= H) return;
    float run = 0.f;
    for (int b = nblk - 1; b >= 0; --b) {
        const float v = bs[(size_t)b * H + h];
        bs[(size_t)b * H + h] = run;
        run += v;
    }
}

// u_i^h = dt_i^h * exp(A^h * (sum of dt over the later tokens of the block + over the later blocks))
__global__ __launch_bounds__(kThreads) void full_prep_apply_kernel(const float *__restrict__ dt,
                                                                   const float *__restrict__ A,
                                                                   const float *__restrict__ bs, float *__restrict__ U,
                                                                   int N, int H, int nblk) {
    const int h = blockIdx.y * kThreads + threadIdx.x;
    if (h >= H) return;
    const int blk = blockIdx.x;
    float run = bs[(size_t)blk * H + h];
    const float a = A[h];
    const int i0 = blk * kRows, i1 = min(N, i0 + kRows);
    for (int i = i1 - 1; i >= i0; --i) {
        const float d = dt[(size_t)i * H + h];
        U[(size_t)i * H + h] = d * __expf(a * run);
        run += d;
    }
}

// One thread per vision token: sum_g sum_m |b_i^g . c_m^g| * sum_{h in g} u_i^h v_m^h.
template <typename T>
__global__ __launch_bounds__(kThreads) void full_score_kernel(const T *__restrict__ Bv, const T *__restrict__ Ct,
                                                              const float *__restrict__ U, const float *__restrict__ V,
                                                              float *__restrict__ s, int M, int N, int H, int G, int n) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    const int hpg = H / G;
    float tot = 0.f;
    for (int g = 0; g < G; ++g) {
        const T *b = Bv + ((size_t)i * G + g) * n;
        const float *u = U + (size_t)i * H + g * hpg;
        for (int m = 0; m < M; ++m) {
            const T *c = Ct + ((size_t)m * G + g) * n;
            float dot = 0.f;
            for (int j = 0; j < n; ++j) dot = fmaf(to_f32(b[j]), to_f32(c[j]), dot);
            const float *v = V + (size_t)m * H + g * hpg;
            float w = 0.f;
            for (int k = 0; k < hpg; ++k) w = fmaf(u[k], v[k], w);
            tot = fmaf(fabsf(dot), w, tot);
        }
    }
    s[i] = tot / ((float)M * (float)H);
}

}  // namespace

// Workspace layout: U [N][H] | V [M][H] | block sums [nblk][H] | group partials (matrix-core path)
static size_t full_u_bytes(int N, int H) { return align_up((size_t)N * H * 4, 256); }
static size_t full_v_bytes(int M, int H) { return align_up((size_t)M * H * 4, 256); }
static size_t full_bs_bytes(int N, int H) { return align_up((size_t)ceil_div(N, kRows) * H * 4, 256); }

size_t score_mamba_full_ws(int M, int N, int H, int G, int n, strd_dtype io) {
    size_t b = full_u_bytes(N, H) + full_v_bytes(M, H) + full_bs_bytes(N, H);
    if (score_mamba_full_mfma_supported(M, N, H, G, n, io)) b += score_mamba_mfma_ws(N, G);
    return b;
}

int score_mamba_full(const void *B, const void *C, const float *dt_all, const float *A, float *s, int M, int N, int H,
                     int G, int n, strd_dtype io, void *ws, hipStream_t st) {
    char *w = (char *)ws;
    float *U = (float *)w;
    float *V = (float *)(w + full_u_bytes(N, H));
    float *bs = (float *)(w + full_u_bytes(N, H) + full_v_bytes(M, H));
    void *part = w + full_u_bytes(N, H) + full_v_bytes(M, H) + full_bs_bytes(N, H);
    const int nblk = ceil_div(N, kRows);
    const dim3 gsum(nblk + 1, ceil_div(H, kThreads)), gapp(nblk, ceil_div(H, kThreads));
    full_prep_sums_kernel<<<gsum, kThreads, 0, st>>>(dt_all, A, bs, V, M, N, H, nblk);
    full_prep_scan_kernel<<<ceil_div(H, kThreads), kThreads, 0, st>>>(bs, H, nblk);
    full_prep_apply_kernel<<<gapp, kThreads, 0, st>>>(dt_all, A, bs, U, N, H, nblk);
    if (score_mamba_full_mfma_supported(M, N, H, G, n, io))
        return score_mamba_full_mfma(B, C, U, V, s, M, N, H, G, n, part, st);
    const int grid = ceil_div(N, kThreads);
    if (io == STRD_F32)
        full_score_kernel<float><<<grid, kThreads, 0, st>>>((const float *)B, (const float *)C, U, V, s, M, N, H, G, n);
    else
        full_score_kernel<bf16_t><<<grid, kThreads, 0, st>>>((const bf16_t *)B, (const bf16_t *)C, U, V, s, M, N, H, G, n);
    return launch_status();
}

}  // namespace strd
