/*
 * strd_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the token-reduced prefill of one
 * hybrid (Mamba-2 / attention) layer computes, written from the paper
 * "Stateful Token Reduction for Long-Video Hybrid VLMs".  Every function is
 * the textbook definition (or the paper's equation) written out as loops; no
 * blocking, fusion or reordering beyond what the cited passage states.  It
 * shares no code with the HIP library and is linked only by the tests, by the
 * smoke check and by the CPU-baseline leg of the benchmark.
 *
 * Conventions (paper Sec. 3.1 and App. "Token Selection via Mamba's Recurrent
 * Updates"): a sequence holds N vision tokens followed by M text tokens; all
 * arrays are token-major, contiguous, double precision.  Head h of H uses
 * group g(h) = h / (H / G) for the shared b, c projections; query head h of Hq
 * uses key/value head h / (Hq / Hkv).  The discretised transition is the
 * scalar a_t = exp(dt_t * A) per head with A < 0, i.e. the paper's
 * exp(-Delta_t A) with its positive A.
 *
 * OpenMP is used only over independent units (query rows, heads, tokens).
 *
 * Parity pins (tests/test_oracle_pins.py): every function below is pinned by
 * closed forms, mutual agreement of independent formulations, brute force on
 * tiny inputs or an independent library routine; nothing here is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Attention importance score (paper Sec. 3.1, "Attention Layers"):   */
/*   s_i = 1/(M*Hq) * sum_{m,h} softmax_i( scale * q_m^h . k_i^kv(h) ) */
/* with the softmax taken over the N vision keys.                     */
/* q: [M,Hq,d]  k: [N,Hkv,d]  s: [N]                                  */
/* ------------------------------------------------------------------ */
int oracle_score_attn(const double *q, const double *k, double *s, int M, int N,
                      int Hq, int Hkv, int d, double scale)
{
    if (M < 1 || N < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv) return -1;
    const int rep = Hq / Hkv;
    for (int i = 0; i < N; ++i) s[i] = 0.0;
    int rc = 0;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)N);
        double *acc = (double *)calloc((size_t)N, sizeof(double));
        if (!z || !acc) {
#pragma omp atomic write
            rc = -2;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int row = 0; row < M * Hq; ++row) {
                const int m = row / Hq, h = row % Hq, hk = h / rep;
                const double *qv = q + ((size_t)m * Hq + h) * d;
                double zmax = -INFINITY;
                for (int i = 0; i < N; ++i) {
                    const double *kv = k + ((size_t)i * Hkv + hk) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += qv[c] * kv[c];
                    z[i] = scale * dot;
                    if (z[i] > zmax) zmax = z[i];
                }
                double denom = 0.0;
                for (int i = 0; i < N; ++i) {
                    z[i] = exp(z[i] - zmax);
                    denom += z[i];
                }
                for (int i = 0; i < N; ++i) acc[i] += z[i] / denom;
            }
#pragma omp critical
            for (int i = 0; i < N; ++i) s[i] += acc[i];
        }
        free(z);
        free(acc);
    }
    if (rc) return rc;
    const double norm = 1.0 / ((double)M * (double)Hq);
    for (int i = 0; i < N; ++i) s[i] *= norm;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Decoupled Content Alignment (paper Eq. "ssm_importance"):          */
/*   s_i = mean over text rows m and heads h of                       */
/*         | (dt_i^h * b_i^{g(h)}) . c_m^{g(h)} |                     */
/* The paper writes the mean over groups with Delta absorbed in b-bar; */
/* Delta is per head in Mamba-2, so the mean runs over every head of   */
/* every group (equal to the group form with the group-mean of Delta). */
/* Bv: [N,G,n]  Ct: [M,G,n]  dtv: [N,H]  s: [N]                        */
/* ------------------------------------------------------------------ */
int oracle_score_mamba(const double *Bv, const double *Ct, const double *dtv,
                       double *s, int M, int N, int H, int G, int n)
{
    if (M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G) return -1;
    const int hpg = H / G;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        double tot = 0.0;
        for (int m = 0; m < M; ++m)
            for (int h = 0; h < H; ++h) {
                const int g = h / hpg;
                const double *b = Bv + ((size_t)i * G + g) * n;
                const double *c = Ct + ((size_t)m * G + g) * n;
                double dot = 0.0;
                for (int j = 0; j < n; ++j) dot += (dtv[(size_t)i * H + h] * b[j]) * c[j];
                tot += fabs(dot);
            }
        s[i] = tot / ((double)M * (double)H);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Full Mamba Dynamic score (paper Eq. "ssm_weight", |w_{t,j}|):       */
/*   s_i = mean_{m,h} | prod_{u=i+1}^{N+m} a_u^h * (dt_i^h b_i).c_m |  */
/* the product running over every position between vision token i and */
/* text row m (text rows sit at positions N..N+M-1).                   */
/* Ball: [N+M,G,n] (only vision rows read)  Call: [N+M,G,n] (only text */
/* rows read)  dt: [N+M,H]  A: [H]  s: [N]                             */
/* ------------------------------------------------------------------ */
/* rows: optional list of nrows vision tokens to score (s then has nrows     */
/* entries, in that order); NULL = all N tokens.                           */
int oracle_score_mamba_full_rows(const double *Ball, const double *Call, const double *dt,
                                 const double *A, double *s, int M, int N, int H, int G, int n,
                                 const int32_t *rows, int nrows)
{
    if (M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G) return -1;
    const int hpg = H / G;
    const int cnt = rows ? nrows : N;
    for (int r = 0; r < cnt; ++r)
        if (rows && (rows[r] < 0 || rows[r] >= N)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < cnt; ++r) {
        const int i = rows ? rows[r] : r;
        double tot = 0.0;
        for (int m = 0; m < M; ++m) {
            const int t = N + m;
            for (int h = 0; h < H; ++h) {
                const int g = h / hpg;
                double decay = 1.0;
                for (int u = i + 1; u <= t; ++u) decay *= exp(dt[(size_t)u * H + h] * A[h]);
                const double *b = Ball + ((size_t)i * G + g) * n;
                const double *c = Call + ((size_t)t * G + g) * n;
                double dot = 0.0;
                for (int j = 0; j < n; ++j) dot += (dt[(size_t)i * H + h] * b[j]) * c[j];
                tot += fabs(decay * dot);
            }
        }
        s[r] = tot / ((double)M * (double)H);
    }
    return 0;
}

int oracle_score_mamba_full(const double *Ball, const double *Call, const double *dt,
                            const double *A, double *s, int M, int N, int H, int G, int n)
{
    return oracle_score_mamba_full_rows(Ball, Call, dt, A, s, M, N, H, G, n, NULL, 0);
}

/* ------------------------------------------------------------------ */
/* Top-K selection preserving temporal order (paper Sec. 3.1, "Token   */
/* Selection"): full stable sort by (score descending, index ascending),*/
/* keep the first K, return their indices ascending.                   */
/* ------------------------------------------------------------------ */
typedef struct { double s; int32_t i; } oracle_pair;

static int cmp_score_desc(const void *a, const void *b)
{
    const oracle_pair *x = (const oracle_pair *)a, *y = (const oracle_pair *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

static int cmp_index_asc(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int oracle_select_topk(const double *s, int N, int K, int32_t *idx)
{
    if (N < 1 || K < 0 || K > N) return -1;
    oracle_pair *p = (oracle_pair *)malloc(sizeof(oracle_pair) * (size_t)N);
    if (!p) return -2;
    for (int i = 0; i < N; ++i) { p[i].s = s[i]; p[i].i = i; }
    qsort(p, (size_t)N, sizeof(oracle_pair), cmp_score_desc);
    for (int r = 0; r < K; ++r) idx[r] = p[r].i;
    qsort(idx, (size_t)K, sizeof(int32_t), cmp_index_asc);
    free(p);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Compaction (paper Sec. 3.1: retained tokens continue, the rest are  */
/* dropped; text tokens are never scored or dropped):                  */
/*   dst[r]   = src[idx[r]]  for r < K                                 */
/*   dst[K+m] = src[N+m]     for m < M                                 */
/* Rows are opaque byte strings; pos (optional) composes index maps.   */
/* ------------------------------------------------------------------ */
int oracle_compact(const void *src, const int32_t *idx, void *dst, int N, int M, int K,
                   int64_t row_bytes, const int32_t *pos_in, int32_t *pos_out)
{
    if (N < 0 || M < 0 || K < 0 || K > N || row_bytes < 0) return -1;
    const char *sp = (const char *)src;
    char *dp = (char *)dst;
    for (int r = 0; r < K; ++r) {
        if (idx[r] < 0 || idx[r] >= N) return -1;
        if (row_bytes) memcpy(dp + (size_t)r * row_bytes, sp + (size_t)idx[r] * row_bytes, (size_t)row_bytes);
        if (pos_out) pos_out[r] = pos_in ? pos_in[idx[r]] : idx[r];
    }
    for (int m = 0; m < M; ++m) {
        if (row_bytes) memcpy(dp + (size_t)(K + m) * row_bytes, sp + (size_t)(N + m) * row_bytes, (size_t)row_bytes);
        if (pos_out) pos_out[K + m] = pos_in ? pos_in[N + m] : N + m;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Mamba-2 recurrence, one token at a time (paper Eqs.                 */
/* "ssm_state_update", "ssm_output"):                                  */
/*   S_t = a_t S_{t-1} + x_t (dt_t b_t)^T,   y_t = S_t c_t (+ D x_t)   */
/* x,y: [T,H,P]  dt: [T,H]  A,D: [H]  B,C: [T,G,n]  S: [H,P,n]         */
/* D, S_in, S_out may be NULL.                                         */
/* ------------------------------------------------------------------ */
int oracle_ssd_seq(const double *x, const double *dt, const double *A, const double *B,
                   const double *C, const double *D, const double *S_in, double *y,
                   double *S_out, int T, int H, int P, int G, int n)
{
    if (T < 0 || H < 1 || P < 1 || G < 1 || n < 1 || H % G) return -1;
    const int hpg = H / G;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        const int g = h / hpg;
        double *S = (double *)calloc((size_t)P * n, sizeof(double));
        if (!S) {
#pragma omp atomic write
            rc = -2;
            continue;
        }
        if (S_in) memcpy(S, S_in + (size_t)h * P * n, sizeof(double) * (size_t)P * n);
        for (int t = 0; t < T; ++t) {
            const double dtt = dt[(size_t)t * H + h];
            const double a = exp(dtt * A[h]);
            const double *b = B + ((size_t)t * G + g) * n;
            const double *c = C + ((size_t)t * G + g) * n;
            const double *xt = x + ((size_t)t * H + h) * P;
            double *yt = y + ((size_t)t * H + h) * P;
            for (int p = 0; p < P; ++p) {
                double out = 0.0;
                for (int j = 0; j < n; ++j) {
                    S[(size_t)p * n + j] = a * S[(size_t)p * n + j] + xt[p] * (dtt * b[j]);
                    out += S[(size_t)p * n + j] * c[j];
                }
                yt[p] = out + (D ? D[h] * xt[p] : 0.0);
            }
        }
        if (S_out) memcpy(S_out + (size_t)h * P * n, S, sizeof(double) * (size_t)P * n);
        free(S);
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* Unrolled / implicit-attention form (paper Eqs. "ssm_unrolled",      */
/* "ssm_attention_form"):                                              */
/*   y_t = sum_{j<=t} ( prod_{u=j+1}^{t} a_u ) (dt_j b_j . c_t) x_j    */
/*         + ( prod_{u=1}^{t} a_u ) S_in c_t                           */
/* O(T^2) per head: small T only.  Products are formed term by term.   */
/* ------------------------------------------------------------------ */
int oracle_ssd_unrolled(const double *x, const double *dt, const double *A, const double *B,
                        const double *C, const double *D, const double *S_in, double *y,
                        int T, int H, int P, int G, int n)
{
    if (T < 0 || H < 1 || P < 1 || G < 1 || n < 1 || H % G) return -1;
    const int hpg = H / G;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        const int g = h / hpg;
        for (int t = 0; t < T; ++t) {
            const double *c = C + ((size_t)t * G + g) * n;
            double *yt = y + ((size_t)t * H + h) * P;
            for (int p = 0; p < P; ++p) yt[p] = 0.0;
            for (int j = 0; j <= t; ++j) {
                double decay = 1.0;
                for (int u = j + 1; u <= t; ++u) decay *= exp(dt[(size_t)u * H + h] * A[h]);
                const double *b = B + ((size_t)j * G + g) * n;
                double dot = 0.0;
                for (int q = 0; q < n; ++q) dot += (dt[(size_t)j * H + h] * b[q]) * c[q];
                const double w = decay * dot;
                const double *xj = x + ((size_t)j * H + h) * P;
                for (int p = 0; p < P; ++p) yt[p] += w * xj[p];
            }
            if (S_in) {
                double decay = 1.0;
                for (int u = 0; u <= t; ++u) decay *= exp(dt[(size_t)u * H + h] * A[h]);
                for (int p = 0; p < P; ++p) {
                    double dot = 0.0;
                    for (int q = 0; q < n; ++q) dot += S_in[((size_t)h * P + p) * n + q] * c[q];
                    yt[p] += decay * dot;
                }
            }
            if (D) {
                const double *xt = x + ((size_t)t * H + h) * P;
                for (int p = 0; p < P; ++p) yt[p] += D[h] * xt[p];
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Chunked form: Eq. "ssm_unrolled" with the sum over j split at chunk */
/* boundaries.  Within a chunk, l_t = sum_{u<=t} dt_u A (u from the    */
/* chunk start);                                                       */
/*   y_t    = sum_{j<=t in chunk} e^{l_t-l_j} (c_t.b_j) dt_j x_j       */
/*            + e^{l_t} S_prev c_t                                     */
/*   S_next = e^{l_Q} S_prev + sum_j e^{l_Q-l_j} dt_j x_j b_j^T        */
/* ------------------------------------------------------------------ */
int oracle_ssd_chunked(const double *x, const double *dt, const double *A, const double *B,
                       const double *C, const double *D, const double *S_in, double *y,
                       double *S_out, int T, int H, int P, int G, int n, int chunk)
{
    if (T < 0 || H < 1 || P < 1 || G < 1 || n < 1 || H % G || chunk < 1) return -1;
    const int hpg = H / G;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        const int g = h / hpg;
        double *S = (double *)calloc((size_t)P * n, sizeof(double));
        double *Sn = (double *)calloc((size_t)P * n, sizeof(double));
        double *l = (double *)calloc((size_t)chunk, sizeof(double));
        if (!S || !Sn || !l) {
#pragma omp atomic write
            rc = -2;
            free(S); free(Sn); free(l);
            continue;
        }
        if (S_in) memcpy(S, S_in + (size_t)h * P * n, sizeof(double) * (size_t)P * n);
        for (int t0 = 0; t0 < T; t0 += chunk) {
            const int Q = (T - t0 < chunk) ? T - t0 : chunk;
            double run = 0.0;
            for (int t = 0; t < Q; ++t) {
                run += dt[(size_t)(t0 + t) * H + h] * A[h];
                l[t] = run;
            }
            for (int t = 0; t < Q; ++t) {
                const double *c = C + ((size_t)(t0 + t) * G + g) * n;
                double *yt = y + ((size_t)(t0 + t) * H + h) * P;
                for (int p = 0; p < P; ++p) {
                    double dot = 0.0;
                    for (int q = 0; q < n; ++q) dot += S[(size_t)p * n + q] * c[q];
                    yt[p] = exp(l[t]) * dot;
                }
                for (int j = 0; j <= t; ++j) {
                    const double *b = B + ((size_t)(t0 + j) * G + g) * n;
                    double cb = 0.0;
                    for (int q = 0; q < n; ++q) cb += c[q] * b[q];
                    const double w = exp(l[t] - l[j]) * cb * dt[(size_t)(t0 + j) * H + h];
                    const double *xj = x + ((size_t)(t0 + j) * H + h) * P;
                    for (int p = 0; p < P; ++p) yt[p] += w * xj[p];
                }
                if (D) {
                    const double *xt = x + ((size_t)(t0 + t) * H + h) * P;
                    for (int p = 0; p < P; ++p) yt[p] += D[h] * xt[p];
                }
            }
            for (size_t e = 0; e < (size_t)P * n; ++e) Sn[e] = exp(l[Q - 1]) * S[e];
            for (int j = 0; j < Q; ++j) {
                const double *b = B + ((size_t)(t0 + j) * G + g) * n;
                const double *xj = x + ((size_t)(t0 + j) * H + h) * P;
                const double w = exp(l[Q - 1] - l[j]) * dt[(size_t)(t0 + j) * H + h];
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < n; ++q) Sn[(size_t)p * n + q] += w * xj[p] * b[q];
            }
            memcpy(S, Sn, sizeof(double) * (size_t)P * n);
        }
        if (S_out) memcpy(S_out + (size_t)h * P * n, S, sizeof(double) * (size_t)P * n);
        free(S); free(Sn); free(l);
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* Causal softmax attention with grouped-query heads (paper App.,      */
/* "Attention via Kernel Functions", first equation):                  */
/*   o_t^h = sum_{j<=t} softmax_j( scale q_t^h . k_j^kv(h) ) v_j^kv(h) */
/* Only the rows listed in `rows` are produced (rows == NULL: all T).  */
/* q: [T,Hq,d]  k,v: [T,Hkv,d]  o: [nrows,Hq,d]                        */
/* ------------------------------------------------------------------ */
int oracle_attn(const double *q, const double *k, const double *v, double *o, int T, int Hq,
                int Hkv, int d, double scale, const int32_t *rows, int nrows)
{
    if (T < 0 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv) return -1;
    if (!rows) nrows = T;
    const int rep = Hq / Hkv;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int r = 0; r < nrows; ++r)
        for (int h = 0; h < Hq; ++h) {
            const int t = rows ? rows[r] : r;
            if (t < 0 || t >= T) {
#pragma omp atomic write
                rc = -1;
                continue;
            }
            const int hk = h / rep;
            const double *qv = q + ((size_t)t * Hq + h) * d;
            double *z = (double *)malloc(sizeof(double) * (size_t)(t + 1));
            if (!z) {
#pragma omp atomic write
                rc = -2;
                continue;
            }
            double zmax = -INFINITY;
            for (int j = 0; j <= t; ++j) {
                const double *kv = k + ((size_t)j * Hkv + hk) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += qv[c] * kv[c];
                z[j] = scale * dot;
                if (z[j] > zmax) zmax = z[j];
            }
            double denom = 0.0;
            for (int j = 0; j <= t; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
            double *ov = o + ((size_t)r * Hq + h) * d;
            for (int c = 0; c < d; ++c) ov[c] = 0.0;
            for (int j = 0; j <= t; ++j) {
                const double w = z[j] / denom;
                const double *vv = v + ((size_t)j * Hkv + hk) * d;
                for (int c = 0; c < d; ++c) ov[c] += w * vv[c];
            }
            free(z);
        }
    return rc;
}

/* ------------------------------------------------------------------ */
/* Block glue (the Mamba-2 block's operations around the scan; the      */
/* paper builds on that block without restating them).                  */
/* ------------------------------------------------------------------ */
static double oracle_silu(double v) { return v / (1.0 + exp(-v)); }

/* out[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + eps) * w */
int oracle_rmsnorm(const double *x, const double *w, double *out, int T, int d, double eps)
{
    if (T < 0 || d < 1) return -1;
    for (int t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) ss += x[(size_t)t * d + c] * x[(size_t)t * d + c];
        const double inv = 1.0 / sqrt(ss / d + eps);
        for (int c = 0; c < d; ++c) out[(size_t)t * d + c] = x[(size_t)t * d + c] * inv * w[c];
    }
    return 0;
}

/* v = y * silu(z); per group of D/groups channels: out = v / sqrt(mean(v^2) + eps) * w */
int oracle_gated_rmsnorm(const double *y, const double *z, const double *w, double *out, int T, int D,
                         int groups, double eps)
{
    if (T < 0 || D < 1 || groups < 1 || D % groups) return -1;
    const int gs = D / groups;
    for (int t = 0; t < T; ++t)
        for (int g = 0; g < groups; ++g) {
            const size_t o = (size_t)t * D + (size_t)g * gs;
            double ss = 0.0;
            for (int c = 0; c < gs; ++c) {
                const double v = y[o + c] * oracle_silu(z[o + c]);
                ss += v * v;
            }
            const double inv = 1.0 / sqrt(ss / gs + eps);
            for (int c = 0; c < gs; ++c) out[o + c] = y[o + c] * oracle_silu(z[o + c]) * inv * w[(size_t)g * gs + c];
        }
    return 0;
}

/* causal depthwise convolution with zero history, then SiLU:                     */
/*   out[t,c] = silu(b[c] + sum_{k<W} w[c,k] * in[t-(W-1)+k, c]),  in, out [T,C]   */
int oracle_conv1d_silu(const double *in, const double *w, const double *b, double *out, int T, int C, int W)
{
    if (T < 0 || C < 1 || W < 1) return -1;
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < C; ++c) {
            double acc = b ? b[c] : 0.0;
            for (int k = 0; k < W; ++k) {
                const int ts = t - (W - 1) + k;
                if (ts >= 0) acc += w[(size_t)c * W + k] * in[(size_t)ts * C + c];
            }
            out[(size_t)t * C + c] = oracle_silu(acc);
        }
    return 0;
}

/* dt[t,h] = log(1 + exp(raw[t,h] + bias[h])) */
int oracle_softplus_dt(const double *raw, const double *bias, double *dt, int T, int H)
{
    if (T < 0 || H < 1) return -1;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h) {
            const double v = raw[(size_t)t * H + h] + (bias ? bias[h] : 0.0);
            dt[(size_t)t * H + h] = v > 0 ? v + log1p(exp(-v)) : log1p(exp(v));
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Average-pool reduction (the baseline the paper's "Reduction Types"  */
/* ablation sets against query-based selection): the N vision rows are */
/* cut into K consecutive windows, window j = rows [floor(j N / K),     */
/* floor((j+1) N / K)), each replaced by its mean; the M text rows      */
/* follow unchanged.  A pooled token takes the position of the first    */
/* row of its window.  The paper does not state the window shape; this  */
/* is the non-overlapping 1-D pooling along the token axis.             */
/* src: [N+M,D]  dst: [K+M,D]  pos_in: [N+M] or NULL  pos_out: [K+M]    */
/* ------------------------------------------------------------------ */
int oracle_avgpool(const double *src, double *dst, int N, int M, int K, int D,
                   const int32_t *pos_in, int32_t *pos_out)
{
    if (N < 0 || M < 0 || K < 0 || K > N || D < 0 || (N > 0 && K == 0)) return -1;
    for (int j = 0; j < K; ++j) {
        const int lo = (int)(((long long)j * N) / K), hi = (int)(((long long)(j + 1) * N) / K);
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int r = lo; r < hi; ++r) acc += src[(size_t)r * D + c];
            dst[(size_t)j * D + c] = acc / (double)(hi - lo);
        }
        if (pos_out) pos_out[j] = pos_in ? pos_in[lo] : lo;
    }
    for (int m = 0; m < M; ++m) {
        for (int c = 0; c < D; ++c) dst[(size_t)(K + m) * D + c] = src[(size_t)(N + m) * D + c];
        if (pos_out) pos_out[K + m] = pos_in ? pos_in[N + m] : N + m;
    }
    return 0;
}
