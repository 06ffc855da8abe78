// General-shape SIMT kernels: fp32 arithmetic on fp32 or bf16 tensors, any head count, head
// dimension and state size.  They serve fp32 I/O (where the 1e-4 tolerance rules out bf16
// matrix cores) and the shapes the MFMA kernels are not tiled for.  Each kernel is the
// definition evaluated directly; the tuned bf16 paths live in the *_mfma.hip files.
#include "common.h"

namespace strd {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// ------------------------------------------------------------------ score_attn -------------
// Pass 1: one workgroup per (text row m, query head h): log-sum-exp of scale * q.k_i over the
// N vision keys.  lse index = m * Hq + h.
// SEQ = SeqTab (packed batch, blockIdx.y = sequence): q and k both point at the packed tensors,
// lse has `lse_ld` entries per sequence.
template <typename T, class SEQ>
__global__ __launch_bounds__(kThreads) void attn_row_lse_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                float *__restrict__ lse, int N, int Hq, int Hkv,
                                                                int d, float scale, SEQ seq, int lse_ld) {
    extern __shared__ float smem[];  // d floats of q, then 2 * waves
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        N = seq.N[b];
        if ((int)blockIdx.x >= seq.M[b] * Hq) return;  // uniform
        k += (size_t)seq.row0[b] * Hkv * d;
        q += (size_t)(seq.row0[b] + N) * Hq * d;
        lse += (size_t)b * lse_ld;
    }
    const int row = blockIdx.x, h = row % Hq, hk = h / (Hq / Hkv);
    float *qs = smem;
    float *red = smem + d;
    for (int c = threadIdx.x; c < d; c += kThreads) qs[c] = to_f32(q[(size_t)row * d + c]);
    __syncthreads();
    float mx = -INFINITY, sum = 0.f;
    for (int i = threadIdx.x; i < N; i += kThreads) {
        const T *kv = k + ((size_t)i * Hkv + hk) * d;
        float dot = 0.f;
        for (int c = 0; c < d; ++c) dot = fmaf(qs[c], to_f32(kv[c]), dot);
        const float z = scale * dot;
        const float nm = fmaxf(mx, z);
        sum = sum * expf(mx - nm) + expf(z - nm);
        mx = nm;
    }
    // combine (max, sum) pairs: wave, then workgroup
    const float wm = wave_max(mx);
    const float ws = wave_sum(mx == -INFINITY ? 0.f : sum * expf(mx - wm));
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (lane == 0) { red[2 * wave] = wm; red[2 * wave + 1] = ws; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float gm = -INFINITY;
        for (int w = 0; w < kThreads / kWave; ++w) gm = fmaxf(gm, red[2 * w]);
        float gs = 0.f;
        for (int w = 0; w < kThreads / kWave; ++w)
            if (red[2 * w] != -INFINITY) gs += red[2 * w + 1] * expf(red[2 * w] - gm);
        lse[row] = gm + logf(gs);
    }
}

// Pass 2: one thread per vision token: sum over all (m, h) rows of exp(z - lse).
template <typename T, class SEQ>
__global__ __launch_bounds__(kThreads) void attn_col_sum_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                const float *__restrict__ lse,
                                                                float *__restrict__ s, int M, int N, int Hq,
                                                                int Hkv, int d, float scale, SEQ seq, int lse_ld,
                                                                int ld) {
    if constexpr (is_varlen<SEQ>()) {
        const int b = blockIdx.y;
        N = seq.N[b];
        M = seq.M[b];
        k += (size_t)seq.row0[b] * Hkv * d;
        q += (size_t)(seq.row0[b] + N) * Hq * d;
        lse += (size_t)b * lse_ld;
        s += (size_t)b * ld;
    }
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    const int rep = Hq / Hkv;
    float acc = 0.f;
    for (int m = 0; m < M; ++m)
        for (int h = 0; h < Hq; ++h) {
            const T *qv = q + ((size_t)m * Hq + h) * d;
            const T *kv = k + ((size_t)i * Hkv + h / rep) * d;
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot = fmaf(to_f32(qv[c]), to_f32(kv[c]), dot);
            acc += expf(scale * dot - lse[m * Hq + h]);
        }
    s[i] = acc / ((float)M * (float)Hq);
}

// ------------------------------------------------------------------ score_mamba ------------
// One thread per vision token: sum_g (sum_{h in g} dt_i^h) * sum_m |b_i^g . c_m^g|.
template <typename T, class SEQ>
__global__ __launch_bounds__(kThreads) void mamba_score_kernel(const T *__restrict__ Bv, const T *__restrict__ Ct,
                                                               const float *__restrict__ dtv,
                                                               float *__restrict__ s, int M, int N, int H, int G,
                                                               int n, SEQ seq, int ld) {
    if constexpr (is_varlen<SEQ>()) {  // blockIdx.y = sequence; Bv, Ct, dtv are the packed tensors
        const int b = blockIdx.y;
        N = seq.N[b];
        M = seq.M[b];
        Bv += (size_t)seq.row0[b] * G * n;
        Ct += (size_t)(seq.row0[b] + N) * G * n;
        dtv += (size_t)seq.row0[b] * H;
        s += (size_t)b * ld;
    }
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    const int hpg = H / G;
    float tot = 0.f;
    for (int g = 0; g < G; ++g) {
        float dts = 0.f;
        for (int h = g * hpg; h < (g + 1) * hpg; ++h) dts += dtv[(size_t)i * H + h];
        const T *b = Bv + ((size_t)i * G + g) * n;
        float a = 0.f;
        for (int m = 0; m < M; ++m) {
            const T *c = Ct + ((size_t)m * G + g) * n;
            float dot = 0.f;
            for (int j = 0; j < n; ++j) dot = fmaf(to_f32(b[j]), to_f32(c[j]), dot);
            a += fabsf(dot);
        }
        tot += dts * a;
    }
    s[i] = tot / ((float)M * (float)H);
}

// ------------------------------------------------------------------ ssd (recurrence) -------
// Token-by-token recurrence.  A state column (h, p) is held by `lanes` adjacent lanes, each
// with kSlice consecutive state entries in registers; y_t is reduced across those lanes.
constexpr int kSlice = 16;

template <typename T>
__global__ __launch_bounds__(kThreads) void ssd_recurrence_kernel(
    const T *__restrict__ x, const float *__restrict__ dt, const float *__restrict__ A, const T *__restrict__ B,
    const T *__restrict__ C, const float *__restrict__ D, const float *__restrict__ S_in, T *__restrict__ y,
    float *__restrict__ S_out, int Tn, int H, int P, int G, int n, int lanes) {
    const int gid = blockIdx.x * kThreads + threadIdx.x;
    const int col = gid / lanes, sub = gid % lanes;
    const bool live = col < H * P;
    const int h = live ? col / P : 0, p = live ? col % P : 0, g = h / (H / G);
    const int j0 = sub * kSlice;
    float S[kSlice];
#pragma unroll
    for (int e = 0; e < kSlice; ++e)
        S[e] = (live && S_in && j0 + e < n) ? S_in[((size_t)h * P + p) * n + j0 + e] : 0.f;
    const float Ah = A[h];
    const float Dh = D ? D[h] : 0.f;
    for (int t = 0; t < Tn; ++t) {
        const float dtt = dt[(size_t)t * H + h];
        const float a = expf(dtt * Ah);
        const float xv = to_f32(x[((size_t)t * H + h) * P + p]);
        const T *b = B + ((size_t)t * G + g) * n + j0;
        const T *c = C + ((size_t)t * G + g) * n + j0;
        float out = 0.f;
#pragma unroll
        for (int e = 0; e < kSlice; ++e)
            if (j0 + e < n) {
                S[e] = a * S[e] + xv * (dtt * to_f32(b[e]));
                out = fmaf(S[e], to_f32(c[e]), out);
            }
        for (int o = lanes / 2; o > 0; o >>= 1) out += __shfl_xor(out, o, kWave);
        if (live && sub == 0) y[((size_t)t * H + h) * P + p] = from_f32<T>(out + Dh * xv);
    }
    if (live && S_out)
#pragma unroll
        for (int e = 0; e < kSlice; ++e)
            if (j0 + e < n) S_out[((size_t)h * P + p) * n + j0 + e] = S[e];
}

// ------------------------------------------------------------------ attention --------------
// One workgroup per (query row t, query head h); keys are walked in tiles of kThreads with an
// online softmax; lane c < d accumulates output channel c.
template <typename T>
__global__ __launch_bounds__(kThreads) void attn_row_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                            const T *__restrict__ v, T *__restrict__ o, int Hq,
                                                            int Hkv, int d, float scale) {
    extern __shared__ float smem[];  // d (q) + kThreads (p) + waves (red)
    float *qs = smem, *ps = smem + d, *red = smem + d + kThreads;
    const int t = blockIdx.x / Hq, h = blockIdx.x % Hq, hk = h / (Hq / Hkv);
    for (int c = threadIdx.x; c < d; c += kThreads) qs[c] = to_f32(q[((size_t)t * Hq + h) * d + c]);
    __syncthreads();
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;  // acc: channel threadIdx.x (< d)
    for (int j0 = 0; j0 <= t; j0 += kThreads) {
        const int j = j0 + threadIdx.x;
        float z = -INFINITY;
        if (j <= t) {
            const T *kv = k + ((size_t)j * Hkv + hk) * d;
            float dot = 0.f;
            for (int c = 0; c < d; ++c) dot = fmaf(qs[c], to_f32(kv[c]), dot);
            z = scale * dot;
        }
        const float wm = wave_max(z);
        if (lane == 0) red[wave] = wm;
        __syncthreads();
        float tm = -INFINITY;
        for (int w = 0; w < kThreads / kWave; ++w) tm = fmaxf(tm, red[w]);
        const float m_new = fmaxf(m_run, tm);
        const float pj = (j <= t) ? expf(z - m_new) : 0.f;
        ps[threadIdx.x] = pj;
        const float wsum = wave_sum(pj);
        __syncthreads();  // ps complete, red (max) consumed
        if (lane == 0) red[wave] = wsum;
        __syncthreads();
        float tsum = 0.f;
        for (int w = 0; w < kThreads / kWave; ++w) tsum += red[w];
        const float corr = expf(m_run - m_new);  // 0 on the first tile (m_run = -inf)
        l_run = l_run * corr + tsum;
        m_run = m_new;
        if (threadIdx.x < d) {
            acc *= corr;
            const int cnt = min(kThreads, t + 1 - j0);
            for (int jj = 0; jj < cnt; ++jj)
                acc = fmaf(ps[jj], to_f32(v[((size_t)(j0 + jj) * Hkv + hk) * d + threadIdx.x]), acc);
        }
        __syncthreads();  // before ps / red are overwritten
    }
    if (threadIdx.x < d) o[((size_t)t * Hq + h) * d + threadIdx.x] = from_f32<T>(acc / l_run);
}

}  // namespace

// ------------------------------------------------------------------ host launchers ---------
size_t score_attn_general_ws(int M, int Hq) { return align_up((size_t)M * Hq * sizeof(float), 256); }

template <typename T, class SEQ>
static void score_attn_launch(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, int d, float scale,
                              float *lse, size_t sm, const SEQ &seq, int nseq, int ld, hipStream_t st) {
    attn_row_lse_kernel<T, SEQ><<<dim3(M * Hq, nseq), kThreads, sm, st>>>((const T *)q, (const T *)k, lse, N, Hq, Hkv, d,
                                                                         scale, seq, M * Hq);
    attn_col_sum_kernel<T, SEQ><<<dim3(ceil_div(N, kThreads), nseq), kThreads, 0, st>>>((const T *)q, (const T *)k, lse, s,
                                                                                      M, N, Hq, Hkv, d, scale, seq,
                                                                                      M * Hq, ld);
}

int score_attn_general(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, int d,
                       float scale, strd_dtype io, void *ws, hipStream_t st) {
    const size_t sm = (size_t)(d + 2 * (kThreads / kWave)) * sizeof(float);
    if (sm > 60000) return STRD_EUNSUPPORTED;
    if (io == STRD_F32)
        score_attn_launch<float>(q, k, s, M, N, Hq, Hkv, d, scale, (float *)ws, sm, OneSeq(), 1, 0, st);
    else
        score_attn_launch<bf16_t>(q, k, s, M, N, Hq, Hkv, d, scale, (float *)ws, sm, OneSeq(), 1, 0, st);
    return launch_status();
}

// Packed batch: grids sized for the longest sequence, lse of sequence b at ws + b * max_m * Hq floats.
int score_attn_general_varlen(const void *q, const void *k, float *s, int ld, const SeqTab &tab, int nseq, int max_m,
                              int max_n, int Hq, int Hkv, int d, float scale, strd_dtype io, void *ws, hipStream_t st) {
    const size_t sm = (size_t)(d + 2 * (kThreads / kWave)) * sizeof(float);
    if (sm > 60000) return STRD_EUNSUPPORTED;
    if (io == STRD_F32)
        score_attn_launch<float>(q, k, s, max_m, max_n, Hq, Hkv, d, scale, (float *)ws, sm, tab, nseq, ld, st);
    else
        score_attn_launch<bf16_t>(q, k, s, max_m, max_n, Hq, Hkv, d, scale, (float *)ws, sm, tab, nseq, ld, st);
    return launch_status();
}

int score_mamba_general(const void *B, const void *C, const float *dt, float *s, int M, int N, int H,
                        int G, int n, strd_dtype io, hipStream_t st) {
    const int grid = ceil_div(N, kThreads);
    if (io == STRD_F32)
        mamba_score_kernel<float, OneSeq><<<grid, kThreads, 0, st>>>((const float *)B, (const float *)C, dt, s, M, N, H, G, n,
                                                                     OneSeq(), 0);
    else
        mamba_score_kernel<bf16_t, OneSeq><<<grid, kThreads, 0, st>>>((const bf16_t *)B, (const bf16_t *)C, dt, s, M, N, H, G,
                                                                      n, OneSeq(), 0);
    return launch_status();
}

int score_mamba_general_varlen(const void *B, const void *C, const float *dt, float *s, int ld, const SeqTab &tab, int nseq, int max_n,
                               int H, int G, int n, strd_dtype io, hipStream_t st) {
    const dim3 grid(ceil_div(max_n, kThreads), nseq);
    if (io == STRD_F32)
        mamba_score_kernel<float, SeqTab><<<grid, kThreads, 0, st>>>((const float *)B, (const float *)C, dt, s, 0, 0, H, G, n,
                                                                     tab, ld);
    else
        mamba_score_kernel<bf16_t, SeqTab><<<grid, kThreads, 0, st>>>((const bf16_t *)B, (const bf16_t *)C, dt, s, 0, 0, H, G,
                                                                      n, tab, ld);
    return launch_status();
}

bool ssd_general_supported(int n) { return n >= 1 && n <= kSlice * kWave; }

int ssd_general(const void *x, const float *dt, const float *A, const void *B, const void *C,
                const float *D, const float *S_in, void *y, float *S_out, int T, int H, int P, int G,
                int n, strd_dtype io, hipStream_t st) {
    int lanes = 1;
    while (lanes * kSlice < n) lanes <<= 1;  // power of two <= 64, so a column never straddles a wave
    const long long threads = (long long)H * P * lanes;
    if (threads > (1LL << 30)) return STRD_EUNSUPPORTED;
    const int grid = (int)((threads + kThreads - 1) / kThreads);
    if (io == STRD_F32)
        ssd_recurrence_kernel<float><<<grid, kThreads, 0, st>>>((const float *)x, dt, A, (const float *)B, (const float *)C, D, S_in, (float *)y, S_out, T, H, P, G, n, lanes);
    else
        ssd_recurrence_kernel<bf16_t><<<grid, kThreads, 0, st>>>((const bf16_t *)x, dt, A, (const bf16_t *)B, (const bf16_t *)C, D, S_in, (bf16_t *)y, S_out, T, H, P, G, n, lanes);
    return launch_status();
}

bool attn_general_supported(int d) { return d >= 1 && d <= kThreads; }

int attn_general(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d,
                 float scale, strd_dtype io, hipStream_t st) {
    if (T == 0) return STRD_OK;
    if ((long long)T * Hq > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    const size_t sm = (size_t)(d + kThreads + kThreads / kWave) * sizeof(float);
    if (io == STRD_F32)
        attn_row_kernel<float><<<T * Hq, kThreads, sm, st>>>((const float *)q, (const float *)k, (const float *)v, (float *)o, Hq, Hkv, d, scale);
    else
        attn_row_kernel<bf16_t><<<T * Hq, kThreads, sm, st>>>((const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, (bf16_t *)o, Hq, Hkv, d, scale);
    return launch_status();
}

}  // namespace strd
