// C ABI of the library: argument checks, workspace accounting and kernel selection.
// Every entry point validates on the host, then enqueues kernels on the caller's stream.
#include <math.h>

#include <string.h>

#include <algorithm>

#include "common.h"

using namespace strd;

namespace {

inline bool io_ok(strd_dtype io) { return io == STRD_F32 || io == STRD_BF16; }
inline hipStream_t as_stream(void *s) { return (hipStream_t)s; }
// The two matrix-core kernels of the scan: segments of the sequence side by side (ssd_seg) where that
// pays, one workgroup per (head, 32 channels) over the whole sequence (ssd_mfma) otherwise.
inline bool use_seg(int T, int rows, int H, int P, int G, int n, strd_dtype io) {
    return ssd_seg_supported(T, rows, H, P, G, n, io) &&
           (ssd_seg_preferred(T, H, P, G) || !ssd_mfma_supported(T, rows, H, P, G, n, io));
}
// The kernels read and write 16-byte vectors straight from the caller's pointers.
template <typename... P>
inline bool aligned16(const P *...p) { return ((... | (uintptr_t)p) & 15u) == 0; }

}  // namespace

extern "C" {

const char *strd_status_string(int status) {
    switch (status) {
        case STRD_OK: return "STRD_OK";
        case STRD_EINVAL: return "STRD_EINVAL: inconsistent arguments";
        case STRD_EUNSUPPORTED: return "STRD_EUNSUPPORTED: no kernel for this shape";
        case STRD_EWORKSPACE: return "STRD_EWORKSPACE: workspace missing or too small";
        case STRD_EHIP: return "STRD_EHIP: HIP launch failed";
        default: return "unknown strd status";
    }
}

int strd_version(void) { return 1000; }

// ------------------------------------------------------------------ score_attn -------------
size_t strd_score_attn_workspace(int M, int N, int Hq, int Hkv, int d, strd_dtype io) {
    if (M < 1 || N < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv) return 0;
    if (score_attn_mfma_supported(M, N, Hq, Hkv, d, io)) return score_attn_mfma_ws(M, N, Hq, Hkv);
    return score_attn_general_ws(M, Hq);
}

int strd_score_attn(const void *q_txt, const void *k_vis, float *scores, int M, int N, int Hq, int Hkv,
                    int d, float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!q_txt || !k_vis || !scores || M < 1 || N < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io) ||
        !(scale > 0.f))
        return STRD_EINVAL;
    if ((long long)M * Hq > (1 << 30)) return STRD_EUNSUPPORTED;
    if (score_attn_mfma_supported(M, N, Hq, Hkv, d, io) && !aligned16(q_txt, k_vis, scores, ws)) return STRD_EINVAL;
    const size_t need = strd_score_attn_workspace(M, N, Hq, Hkv, d, io);
    if (!ws || ws_bytes < need) return STRD_EWORKSPACE;
    if (score_attn_mfma_supported(M, N, Hq, Hkv, d, io))
        return score_attn_mfma(q_txt, k_vis, scores, M, N, Hq, Hkv, d, scale, ws, as_stream(stream));
    return score_attn_general(q_txt, k_vis, scores, M, N, Hq, Hkv, d, scale, io, ws, as_stream(stream));
}

// ------------------------------------------------------------------ score_mamba ------------
size_t strd_score_mamba_workspace(int M, int N, int H, int G, int n, strd_dtype io) {
    if (M < 1 || N < 1 || H < 1 || G < 1 || H % G) return 0;
    return score_mamba_mfma_supported(M, N, H, G, n, io) ? score_mamba_mfma_ws(N, G) : 0;
}

int strd_score_mamba(const void *B_vis, const void *C_txt, const float *dt_vis, float *scores, int M, int N,
                     int H, int G, int n, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!B_vis || !C_txt || !dt_vis || !scores || M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G || !io_ok(io))
        return STRD_EINVAL;
    if (score_mamba_mfma_supported(M, N, H, G, n, io) && !aligned16(B_vis, C_txt, dt_vis, scores, ws)) return STRD_EINVAL;
    const size_t need = strd_score_mamba_workspace(M, N, H, G, n, io);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    if (score_mamba_mfma_supported(M, N, H, G, n, io))
        return score_mamba_mfma(B_vis, C_txt, dt_vis, scores, M, N, H, G, n, ws, as_stream(stream));
    return score_mamba_general(B_vis, C_txt, dt_vis, scores, M, N, H, G, n, io, as_stream(stream));
}

size_t strd_score_mamba_full_workspace(int M, int N, int H, int G, int n, strd_dtype io) {
    if (M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G) return 0;
    return score_mamba_full_ws(M, N, H, G, n, io);
}

int strd_score_mamba_full(const void *B_vis, const void *C_txt, const float *dt_all, const float *A, float *scores,
                          int M, int N, int H, int G, int n, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!B_vis || !C_txt || !dt_all || !A || !scores || M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G || !io_ok(io))
        return STRD_EINVAL;
    if (score_mamba_full_mfma_supported(M, N, H, G, n, io) && !aligned16(B_vis, C_txt, dt_all, scores, ws)) return STRD_EINVAL;
    if ((long long)N + M > 0x7FFFFFFFLL || H > 65535 * 256) return STRD_EUNSUPPORTED;
    const size_t need = strd_score_mamba_full_workspace(M, N, H, G, n, io);
    if (!ws || ws_bytes < need) return STRD_EWORKSPACE;
    return score_mamba_full(B_vis, C_txt, dt_all, A, scores, M, N, H, G, n, io, ws, as_stream(stream));
}

// ------------------------------------------------------------------ select_topk ------------
size_t strd_select_topk_workspace(int N, int K) {
    (void)K;
    return N >= 1 ? select_topk_ws(N) : 0;
}

int strd_select_topk(const float *scores, int N, int K, int32_t *idx, void *ws, size_t ws_bytes, void *stream) {
    if (!scores || !idx || N < 1 || K < 1 || K > N || !aligned16(scores, ws)) return STRD_EINVAL;
    if (N > (1 << 30)) return STRD_EUNSUPPORTED;
    const size_t need = select_topk_ws(N);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    return select_topk_launch(scores, N, K, idx, ws, as_stream(stream));
}

int strd_select_topk_noalloc_max_n(void) { return select_topk_static_max_n(); }

int strd_select_topk_noalloc(const float *scores, int N, int K, int32_t *idx, void *stream) {
    if (!scores || !idx || N < 1 || K < 1 || K > N || !aligned16(scores)) return STRD_EINVAL;
    if (N > select_topk_static_max_n()) return STRD_EUNSUPPORTED;
    return select_topk_static_launch(scores, N, K, idx, as_stream(stream));
}

// ------------------------------------------------------------------ compact ----------------
int strd_compact_batch(const strd_compact_item *items, int n_items, const int32_t *idx, int N, int M, int K,
                       const int32_t *pos_in, int32_t *pos_out, void *stream) {
    if (N < 0 || M < 0 || K < 0 || K > N || (K > 0 && !idx)) return STRD_EINVAL;
    if (n_items < 0 || n_items > STRD_COMPACT_MAX || (n_items > 0 && !items)) return STRD_EINVAL;
    if (n_items == 0 && !pos_out) return STRD_EINVAL;
    for (int i = 0; i < n_items; ++i)
        if (!items[i].src || !items[i].dst || items[i].row_bytes <= 0 || items[i].row_bytes % 4) return STRD_EINVAL;
    if ((long long)K + M > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    return compact_launch(items, n_items, idx, N, M, K, pos_in, pos_out, as_stream(stream));
}

int strd_compact(const void *src, const int32_t *idx, void *dst, int N, int M, int K, int64_t row_bytes,
                 const int32_t *pos_in, int32_t *pos_out, void *stream) {
    if ((src == nullptr) != (dst == nullptr)) return STRD_EINVAL;
    strd_compact_item it = {src, dst, row_bytes};
    return strd_compact_batch(&it, src ? 1 : 0, idx, N, M, K, pos_in, pos_out, stream);
}

// ------------------------------------------------------------------ measurement aid --------
int strd_mfma_rate_probe(float *out, int workgroups, int iters, int mode, void *stream) {
    if (!out || workgroups < 1 || iters < 1 || workgroups > (1 << 20) || mode < 0 || mode > 3) return STRD_EINVAL;
    return mfma_rate_probe(out, workgroups, iters, mode, as_stream(stream));
}

// ------------------------------------------------------------------ packed batches ---------
namespace {
struct SeqPlan {
    SeqTab tab;
    int max_n = 0, max_m = 0, max_out = 0;
    long long rows = 0, kept = 0, out_rows = 0;
};
// Validates the caller's descriptors and lays the sequences out.  K is checked only where it is used.
bool plan_seqs(const strd_seq *seqs, int nseq, bool need_k, SeqPlan &p) {
    if (!seqs || nseq < 1 || nseq > STRD_VARLEN_MAX) return false;
    for (int b = 0; b < nseq; ++b) {
        const strd_seq &q = seqs[b];
        if (q.N < 1 || q.M < 1) return false;
        if (need_k && (q.K < 1 || q.K > q.N)) return false;
        const int k = need_k ? q.K : 0;
        if (p.rows + q.N + q.M > 0x7FFFFFFFLL) return false;
        p.tab.row0[b] = (int)p.rows;
        p.tab.N[b] = q.N;
        p.tab.M[b] = q.M;
        p.tab.K[b] = k;
        p.tab.koff[b] = (int)p.kept;
        p.tab.ooff[b] = (int)p.out_rows;
        p.rows += q.N + q.M;
        p.kept += k;
        p.out_rows += k + q.M;
        p.max_n = std::max(p.max_n, q.N);
        p.max_m = std::max(p.max_m, q.M);
        p.max_out = std::max(p.max_out, k + q.M);
    }
    for (int b = nseq; b < STRD_VARLEN_MAX; ++b)
        p.tab.row0[b] = p.tab.N[b] = p.tab.M[b] = p.tab.K[b] = p.tab.koff[b] = p.tab.ooff[b] = 0;
    return true;
}
}  // namespace

size_t strd_score_attn_varlen_workspace(const strd_seq *seqs, int nseq, int Hq, int Hkv, int d, strd_dtype io) {
    SeqPlan p;
    if (!plan_seqs(seqs, nseq, false, p) || Hq < 1 || Hkv < 1 || Hq % Hkv) return 0;
    if (score_attn_mfma_supported(p.max_m, p.max_n, Hq, Hkv, d, io))
        return score_attn_mfma_varlen_ws(nseq, p.max_m, p.max_n, Hq, Hkv);
    return align_up((size_t)nseq * p.max_m * Hq * sizeof(float), 256);
}

int strd_score_attn_varlen(const void *q_all, const void *k_all, float *scores, int ld, const strd_seq *seqs, int nseq,
                           int Hq, int Hkv, int d, float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    SeqPlan p;
    if (!q_all || !k_all || !scores || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io) ||
        !plan_seqs(seqs, nseq, false, p) || ld < p.max_n || ld % 4 || (long long)p.max_m * Hq > (1 << 30))
        return STRD_EINVAL;
    const bool mfma = score_attn_mfma_supported(p.max_m, p.max_n, Hq, Hkv, d, io);
    if (mfma && !aligned16(q_all, k_all, scores, ws)) return STRD_EINVAL;
    const size_t need = strd_score_attn_varlen_workspace(seqs, nseq, Hq, Hkv, d, io);
    if (!ws || ws_bytes < need) return STRD_EWORKSPACE;
    if (mfma)
        return score_attn_mfma_varlen(q_all, k_all, scores, ld, p.tab, nseq, p.max_m, p.max_n, Hq, Hkv, d, scale, ws,
                                      as_stream(stream));
    return score_attn_general_varlen(q_all, k_all, scores, ld, p.tab, nseq, p.max_m, p.max_n, Hq, Hkv, d, scale, io, ws,
                                     as_stream(stream));
}

size_t strd_score_mamba_varlen_workspace(const strd_seq *seqs, int nseq, int H, int G, int n, strd_dtype io) {
    SeqPlan p;
    if (!plan_seqs(seqs, nseq, false, p) || H < 1 || G < 1 || H % G) return 0;
    return score_mamba_mfma_supported(p.max_m, p.max_n, H, G, n, io) ? align_up((size_t)p.rows * G * sizeof(float), 256) : 0;
}

int strd_score_mamba_varlen(const void *B_all, const void *C_all, const float *dt_all, float *scores, int ld,
                            const strd_seq *seqs, int nseq, int H, int G, int n, strd_dtype io, void *ws, size_t ws_bytes,
                            void *stream) {
    SeqPlan p;
    // b and c are one packed tensor each; the library reads vision rows of B_all and text rows of C_all
    if (!B_all || !C_all || !dt_all || !scores || H < 1 || G < 1 || n < 1 || H % G || !io_ok(io) ||
        !plan_seqs(seqs, nseq, false, p) || ld < p.max_n || ld % 4)
        return STRD_EINVAL;
    const bool mfma = score_mamba_mfma_supported(p.max_m, p.max_n, H, G, n, io);
    if (mfma && !aligned16(B_all, C_all, dt_all, scores, ws)) return STRD_EINVAL;
    const size_t need = strd_score_mamba_varlen_workspace(seqs, nseq, H, G, n, io);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    if (mfma)
        return score_mamba_mfma_varlen(B_all, C_all, dt_all, scores, ld, p.tab, nseq, p.max_n, H, G, n, ws,
                                       as_stream(stream));
    return score_mamba_general_varlen(B_all, C_all, dt_all, scores, ld, p.tab, nseq, p.max_n, H, G, n, io,
                                      as_stream(stream));
}

int strd_select_topk_varlen_max_n(void) { return select_topk_varlen_max_n(); }

int strd_select_topk_varlen(const float *scores, int ld, const strd_seq *seqs, int nseq, int32_t *idx, void *stream) {
    SeqPlan p;
    if (!scores || !idx || !plan_seqs(seqs, nseq, true, p) || ld < p.max_n || ld % 4 || !aligned16(scores))
        return STRD_EINVAL;
    if (p.max_n > select_topk_varlen_max_n()) return STRD_EUNSUPPORTED;
    return select_topk_varlen_launch(scores, ld, p.tab, nseq, p.max_n, idx, as_stream(stream));
}

int strd_compact_varlen(const strd_compact_item *items, int n_items, const int32_t *idx, const strd_seq *seqs, int nseq,
                        const int32_t *pos_in, int32_t *pos_out, void *stream) {
    SeqPlan p;
    if (!idx || !plan_seqs(seqs, nseq, true, p)) return STRD_EINVAL;
    if (n_items < 0 || n_items > STRD_COMPACT_MAX || (n_items > 0 && !items)) return STRD_EINVAL;
    if (n_items == 0 && !pos_out) return STRD_EINVAL;
    for (int i = 0; i < n_items; ++i)
        if (!items[i].src || !items[i].dst || items[i].row_bytes <= 0 || items[i].row_bytes % 4) return STRD_EINVAL;
    if (p.out_rows > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    return compact_varlen_launch(items, n_items, idx, p.tab, nseq, p.max_out, pos_in, pos_out, as_stream(stream));
}

// ------------------------------------------------------------------ ssd_prefill ------------
size_t strd_ssd_prefill_workspace(int T, int H, int P, int G, int n, int chunk, strd_dtype io) {
    (void)chunk;
    if (T < 1 || H < 1 || P < 1 || G < 1 || n < 1 || H % G) return 0;
    return use_seg(T, T, H, P, G, n, io) ? ssd_seg_ws(T, H, P, G, n) : 0;
}

int strd_ssd_prefill(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
                     const float *S_in, void *y, float *S_out, int T, int H, int P, int G, int n, int chunk,
                     strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (T < 0 || H < 1 || P < 1 || G < 1 || n < 1 || H % G || chunk < 1 || !io_ok(io) || !A) return STRD_EINVAL;
    if (T > 0 && (!x || !dt || !B || !C || !y)) return STRD_EINVAL;
    const bool mfma = ssd_mfma_supported(T, T, H, P, G, n, io) || ssd_seg_supported(T, T, H, P, G, n, io);
    if (mfma && !aligned16(x, B, C, S_in, y, S_out, ws)) return STRD_EINVAL;
    const size_t need = strd_ssd_prefill_workspace(T, H, P, G, n, chunk, io);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    if (use_seg(T, T, H, P, G, n, io))
        return ssd_seg(x, dt, A, B, C, D, S_in, y, S_out, nullptr, 0, 0, T, H, P, G, n, ws, as_stream(stream));
    if (mfma) return ssd_mfma(x, dt, A, B, C, D, S_in, y, S_out, nullptr, 0, 0, T, H, P, G, n, as_stream(stream));
    if (!ssd_general_supported(n)) return STRD_EUNSUPPORTED;
    return ssd_general(x, dt, A, B, C, D, S_in, y, S_out, T, H, P, G, n, io, as_stream(stream));
}

int strd_ssd_prefill_gather(const void *x, const float *dt, const float *A, const void *B, const void *C,
                            const float *D, const float *S_in, const int32_t *idx, void *y, float *S_out, int N, int M,
                            int K, int H, int P, int G, int n, int chunk, strd_dtype io, void *ws, size_t ws_bytes,
                            void *stream) {
    if (N < 0 || M < 0 || K < 0 || K > N || H < 1 || P < 1 || G < 1 || n < 1 || H % G || chunk < 1 || !io_ok(io) || !A)
        return STRD_EINVAL;
    const long long T = (long long)K + M;
    if (T > 0 && (!x || !dt || !B || !C || !y || (K > 0 && !idx))) return STRD_EINVAL;
    if (!aligned16(x, B, C, S_in, y, S_out, ws)) return STRD_EINVAL;
    if (T == 0 || (long long)N + M > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    if (!ssd_seg_supported((int)T, N + M, H, P, G, n, io) && !ssd_mfma_supported((int)T, N + M, H, P, G, n, io))
        return STRD_EUNSUPPORTED;
    // the same choice of kernel as strd_ssd_prefill makes for K + M tokens: the results must be the same bits
    const bool old = !use_seg((int)T, (int)T, H, P, G, n, io) || !ssd_seg_supported((int)T, N + M, H, P, G, n, io);
    if (old && !ssd_mfma_supported((int)T, N + M, H, P, G, n, io)) return STRD_EUNSUPPORTED;
    const size_t need = old ? 0 : ssd_seg_ws((int)T, H, P, G, n);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    if (K == 0) {  // only the text rows survive: a dense scan over the tail of the tensors
        const size_t es = 2;
        if (old)
            return ssd_mfma((const char *)x + (size_t)N * H * P * es, dt + (size_t)N * H, A,
                            (const char *)B + (size_t)N * G * n * es, (const char *)C + (size_t)N * G * n * es, D, S_in, y,
                            S_out, nullptr, 0, 0, (int)T, H, P, G, n, as_stream(stream));
        return ssd_seg((const char *)x + (size_t)N * H * P * es, dt + (size_t)N * H, A,
                       (const char *)B + (size_t)N * G * n * es, (const char *)C + (size_t)N * G * n * es, D, S_in, y,
                       S_out, nullptr, 0, 0, (int)T, H, P, G, n, ws, as_stream(stream));
    }
    if (old) return ssd_mfma(x, dt, A, B, C, D, S_in, y, S_out, idx, N, K, (int)T, H, P, G, n, as_stream(stream));
    return ssd_seg(x, dt, A, B, C, D, S_in, y, S_out, idx, N, K, (int)T, H, P, G, n, ws, as_stream(stream));
}

// ------------------------------------------------------------------ attn_prefill -----------
size_t strd_attn_prefill_workspace(int T, int Hq, int Hkv, int d, strd_dtype io) {
    (void)T; (void)Hq; (void)Hkv; (void)d; (void)io;
    return 0;
}

int strd_attn_prefill(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d,
                      float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (T < 0 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io) || !(scale > 0.f)) return STRD_EINVAL;
    if (T > 0 && (!q || !k || !v || !o)) return STRD_EINVAL;
    if (attn_mfma_supported(T, Hq, Hkv, d, io) && !aligned16(q, k, v, o, ws)) return STRD_EINVAL;
    const size_t need = strd_attn_prefill_workspace(T, Hq, Hkv, d, io);
    if (need && (!ws || ws_bytes < need)) return STRD_EWORKSPACE;
    if (attn_mfma_supported(T, Hq, Hkv, d, io)) return attn_mfma(q, k, v, o, T, Hq, Hkv, d, scale, as_stream(stream));
    if (!attn_general_supported(d)) return STRD_EUNSUPPORTED;
    return attn_general(q, k, v, o, T, Hq, Hkv, d, scale, io, as_stream(stream));
}

// ------------------------------------------------------------------ kernel paths -----------
int strd_score_attn_kernel_path(int M, int N, int Hq, int Hkv, int d, strd_dtype io) {
    if (M < 1 || N < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io) || (long long)M * Hq > (1 << 30))
        return STRD_PATH_NONE;
    return score_attn_mfma_supported(M, N, Hq, Hkv, d, io) ? STRD_PATH_MFMA : STRD_PATH_SIMT;
}

int strd_score_mamba_kernel_path(int M, int N, int H, int G, int n, strd_dtype io) {
    if (M < 1 || N < 1 || H < 1 || G < 1 || n < 1 || H % G || !io_ok(io)) return STRD_PATH_NONE;
    return score_mamba_mfma_supported(M, N, H, G, n, io) ? STRD_PATH_MFMA : STRD_PATH_SIMT;
}

int strd_ssd_prefill_kernel_path(int T, int H, int P, int G, int n, strd_dtype io) {
    if (T < 0 || H < 1 || P < 1 || G < 1 || n < 1 || H % G || !io_ok(io)) return STRD_PATH_NONE;
    if (ssd_seg_supported(T, T, H, P, G, n, io) || ssd_mfma_supported(T, T, H, P, G, n, io)) return STRD_PATH_MFMA;
    return ssd_general_supported(n) ? STRD_PATH_SIMT : STRD_PATH_NONE;
}

int strd_attn_prefill_kernel_path(int T, int Hq, int Hkv, int d, strd_dtype io) {
    if (T < 0 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io)) return STRD_PATH_NONE;
    if (attn_mfma_supported(T, Hq, Hkv, d, io)) return STRD_PATH_MFMA;
    return attn_general_supported(d) ? STRD_PATH_SIMT : STRD_PATH_NONE;
}

// ------------------------------------------------------------------ block glue -------------
int strd_rmsnorm(const void *x, const void *w, void *out, int T, int d, float eps, strd_dtype io, void *stream) {
    if (T < 0 || d < 1 || !io_ok(io) || !(eps >= 0.f) || (T > 0 && (!x || !w || !out))) return STRD_EINVAL;
    return glue_rmsnorm(x, w, out, T, d, eps, io, as_stream(stream));
}

int strd_gated_rmsnorm(const void *y, const void *z, int ldz, const void *w, void *out, int T, int D, int groups,
                       float eps, strd_dtype io, void *stream) {
    if (T < 0 || D < 1 || groups < 1 || D % groups || ldz < D || !io_ok(io) || !(eps >= 0.f) ||
        (T > 0 && (!y || !z || !w || !out)))
        return STRD_EINVAL;
    if ((long long)T * groups > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    return glue_gated_rmsnorm(y, z, ldz, w, out, T, D, groups, eps, io, as_stream(stream));
}

int strd_conv1d_silu(const void *xbc, int ld, const void *w, const void *b, void *x_out, void *B_out, void *C_out, int T,
                     int Cx, int Cb, int W, strd_dtype io, void *stream) {
    if (T < 0 || Cx < 0 || Cb < 0 || Cx + 2 * Cb < 1 || W < 1 || ld < Cx + 2 * Cb || !io_ok(io) ||
        (T > 0 && (!xbc || !w || (Cx && !x_out) || (Cb && (!B_out || !C_out)))))
        return STRD_EINVAL;
    // 8-channel vectors: column ranges, row pitch and base addresses must keep them whole and aligned
    const size_t es = io == STRD_F32 ? 4 : 2;
    if (Cx % 8 || Cb % 8 || ld % 8 || ((uintptr_t)xbc % (8 * es)) || ((uintptr_t)x_out % (8 * es)) ||
        ((uintptr_t)B_out % (8 * es)) || ((uintptr_t)C_out % (8 * es)) || ((uintptr_t)w % (8 * es)) ||
        ((uintptr_t)b % (8 * es)))
        return STRD_EUNSUPPORTED;
    if (W > glue_conv_max_width()) return STRD_EUNSUPPORTED;
    if ((long long)T * ((Cx + 2 * Cb) / 8) > 0x7FFFFFFFLL * 256LL) return STRD_EUNSUPPORTED;
    return glue_conv1d_silu(xbc, ld, w, b, x_out, B_out, C_out, T, Cx, Cb, W, io, as_stream(stream));
}

int strd_softplus_dt(const void *raw, int ld, int col0, const float *bias, float *dt, int T, int H, strd_dtype io,
                     void *stream) {
    if (T < 0 || H < 1 || col0 < 0 || ld < col0 + H || !io_ok(io) || (T > 0 && (!raw || !dt))) return STRD_EINVAL;
    return glue_softplus_dt(raw, ld, col0, bias, dt, T, H, io, as_stream(stream));
}

int strd_linear(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, strd_dtype io,
                void *stream) {
    if (T < 0 || Kd < 1 || Nd < 1 || !io_ok(io) || !w || (T > 0 && (!x || !out))) return STRD_EINVAL;
    if (T == 0) return STRD_OK;
    // The library's own kernel where it is at least as fast as the library product: bf16 shapes it is tiled
    // for with a 256 x 256 tile for every CU (measured: equal within 3 % from 272 tiles up, 1.3-2.7x behind
    // below 150).  Everything else -- fp32, odd shapes, small products -- goes to rocBLAS.
    if (linear_mfma_supported(T, Kd, Nd, io) && (long long)ceil_div(T, 256) * ceil_div(Nd, 256) >= 256 &&
        ((((uintptr_t)x | (uintptr_t)w | (uintptr_t)residual | (uintptr_t)out) & 15) == 0))
        return linear_mfma(x, w, residual, out, T, Kd, Nd, as_stream(stream));
    return linear_rocblas(x, w, residual, out, T, Kd, Nd, io, as_stream(stream));
}

int strd_linear_library(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, strd_dtype io,
                        void *stream) {
    if (T < 0 || Kd < 1 || Nd < 1 || !io_ok(io) || !w || (T > 0 && (!x || !out))) return STRD_EINVAL;
    if (T == 0) return STRD_OK;
    return linear_rocblas(x, w, residual, out, T, Kd, Nd, io, as_stream(stream));
}

int strd_linear_mfma_supported(int T, int Kd, int Nd, strd_dtype io) { return linear_mfma_supported(T, Kd, Nd, io) ? 1 : 0; }

int strd_linear_mfma(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, strd_dtype io,
                     void *stream) {
    if (T < 0 || Kd < 1 || Nd < 1 || !io_ok(io) || !w || (T > 0 && (!x || !out))) return STRD_EINVAL;
    if (T == 0) return STRD_OK;
    if (!linear_mfma_supported(T, Kd, Nd, io)) return STRD_EUNSUPPORTED;
    if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)residual | (uintptr_t)out) & 15) return STRD_EINVAL;
    return linear_mfma(x, w, residual, out, T, Kd, Nd, as_stream(stream));
}

// ------------------------------------------------------------------ variants ---------------
int strd_avgpool(const void *src, void *dst, int N, int M, int K, int D, strd_dtype io, const int32_t *pos_in,
                 int32_t *pos_out, void *stream) {
    if (N < 0 || M < 0 || K < 0 || K > N || (N > 0 && K == 0) || D < 0 || !io_ok(io)) return STRD_EINVAL;
    if ((src == nullptr) != (dst == nullptr)) return STRD_EINVAL;
    if ((long long)N + M > 0x7FFFFFFFLL) return STRD_EUNSUPPORTED;
    return avgpool_launch(src, dst, N, M, K, D, io, pos_in, pos_out, as_stream(stream));
}

int strd_ssd_decode_step(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
                         float *S, void *y, int H, int P, int G, int n, strd_dtype io, void *stream) {
    if (H < 1 || P < 1 || G < 1 || n < 1 || H % G || !io_ok(io) || !x || !dt || !A || !B || !C || !S || !y)
        return STRD_EINVAL;
    if ((long long)H * P > (1 << 24)) return STRD_EUNSUPPORTED;
    return ssd_decode_launch(x, dt, A, B, C, D, S, y, H, P, G, n, io, as_stream(stream));
}

size_t strd_attn_decode_step_workspace(int T, int Hq, int Hkv, int d, strd_dtype io) {
    (void)io;
    if (T < 1 || Hq < 1 || Hkv < 1 || d < 1) return 0;
    return attn_decode_workspace(T, Hq, Hkv, d);
}

int strd_attn_decode_step(const void *q, const void *k_cache, const void *v_cache, void *o, int T, int Hq, int Hkv,
                          int d, float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (T < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv || !io_ok(io) || !(scale > 0.f) || !q || !k_cache || !v_cache ||
        !o)
        return STRD_EINVAL;
    if (!attn_decode_supported(Hq, Hkv, d)) return STRD_EUNSUPPORTED;
    const size_t al = 8 * (io == STRD_BF16 ? 2 : 4);
    if ((uintptr_t)q % al || (uintptr_t)k_cache % al || (uintptr_t)v_cache % al) return STRD_EUNSUPPORTED;
    const size_t need = attn_decode_workspace(T, Hq, Hkv, d);
    if (!ws || ws_bytes < need || (uintptr_t)ws % 16) return STRD_EWORKSPACE;
    return attn_decode_launch(q, k_cache, v_cache, o, T, Hq, Hkv, d, scale, io, (float *)ws, as_stream(stream));
}

// ------------------------------------------------------------------ schedules (host) -------
int strd_schedule_budgets(const double *alpha, int L, int N0, int K_min, int32_t *K_out) {
    if (!alpha || !K_out || L < 0 || N0 < 0 || K_min < 0) return STRD_EINVAL;
    long long cur = N0;
    for (int l = 0; l < L; ++l) {
        if (!(alpha[l] >= 0.0 && alpha[l] <= 1.0)) return STRD_EINVAL;
        // the small bias keeps products such as 0.15 * 36864 from landing one below
        // their exact value because alpha is not representable in binary
        long long want = (long long)floor(alpha[l] * (double)N0 + 1e-9);
        const long long floor_k = K_min < cur ? K_min : cur;
        if (want < floor_k) want = floor_k;
        if (want < cur) cur = want;
        K_out[l] = (int32_t)cur;
    }
    return STRD_OK;
}

int strd_schedule_sigmoid(int L, double a_start, double a_end, double k, double x0, double *alpha_out) {
    if (!alpha_out || L < 1) return STRD_EINVAL;
    for (int l = 0; l < L; ++l) {
        const double z = k * (x0 - (double)l / (double)L);
        alpha_out[l] = a_end + (a_start - a_end) / (1.0 + exp(-z));
    }
    return STRD_OK;
}

int strd_schedule_step_decay(const int *lo, const int *hi, const double *alpha, int nranges, int L,
                             double *alpha_out) {
    if (!alpha_out || L < 1 || nranges < 0 || (nranges && (!lo || !hi || !alpha))) return STRD_EINVAL;
    for (int l = 0; l < L; ++l) alpha_out[l] = 1.0;
    for (int r = 0; r < nranges; ++r) {
        if (lo[r] < 0 || hi[r] < lo[r] || hi[r] >= L || !(alpha[r] >= 0.0 && alpha[r] <= 1.0)) return STRD_EINVAL;
        for (int l = lo[r]; l <= hi[r]; ++l) alpha_out[l] = alpha[r];
    }
    return STRD_OK;
}

int strd_hybrid_layout(int L, int32_t *type_out) {
    if (!type_out || L < 1) return STRD_EINVAL;
    int other = 0;
    for (int l = 0; l < L; ++l) {
        if (l >= 7 && (l - 7) % 9 == 0 && l <= 52)
            type_out[l] = STRD_LAYER_ATTN;
        else
            type_out[l] = (other++ % 2 == 0) ? STRD_LAYER_MAMBA : STRD_LAYER_MLP;
    }
    return STRD_OK;
}

int strd_schedule_named(const char *name, double *alpha_out) {
    if (!name || !alpha_out) return STRD_EINVAL;
    const int L = STRD_HYBRID_LAYERS;
    struct Range { int lo, hi; double a; };
    struct Named { const char *name; int n; Range r[7]; };
    static const Named table[] = {
        {"attn_only_1st_attn", 2, {{0, 6, 1.0}, {7, 61, 0.15}}},
        {"all_attn_25", 4, {{0, 6, 1.0}, {7, 15, 0.25}, {16, 33, 0.20}, {34, 61, 0.10}}},
        {"all_attn_35", 6, {{0, 6, 1.0}, {7, 15, 0.50}, {16, 24, 0.40}, {25, 33, 0.30}, {34, 42, 0.20}, {43, 61, 0.10}}},
        {"all_attn_50", 7, {{0, 6, 1.0}, {7, 15, 0.65}, {16, 24, 0.60}, {25, 33, 0.50}, {34, 42, 0.40}, {43, 51, 0.30},
                            {52, 61, 0.20}}},
        {"first_mamba", 1, {{0, 61, 0.25}}},
        {"second_mamba", 2, {{0, 0, 1.0}, {1, 61, 0.23}}},
    };
    for (const Named &t : table) {
        if (strcmp(name, t.name)) continue;
        int lo[7], hi[7];
        double a[7];
        for (int i = 0; i < t.n; ++i) { lo[i] = t.r[i].lo; hi[i] = t.r[i].hi; a[i] = t.r[i].a; }
        return strd_schedule_step_decay(lo, hi, a, t.n, L, alpha_out);
    }
    if (!strcmp(name, "sigmoid_25")) return strd_schedule_sigmoid(L, 1.0, 0.125, 20.0, 0.11, alpha_out);
    if (!strcmp(name, "sigmoid_35")) return strd_schedule_sigmoid(L, 1.0, 0.125, 20.0, 0.24, alpha_out);
    if (!strcmp(name, "sigmoid_50")) return strd_schedule_sigmoid(L, 1.0, 0.125, 20.0, 0.41, alpha_out);
    const int extra = !strcmp(name, "all_attn_1m") ? 1 : !strcmp(name, "all_attn_2m") ? 2 : 0;
    if (extra) {
        // the 6 attention layers reduce, and so do the first `extra` Mamba layers after layer 0 and
        // after every attention layer (6 + 7 reducing layers for extra = 1); the ratio falls linearly
        // from 0.32 at the first reducing layer to 0.15 at the last one up to layer 33, held from there on
        int32_t type[STRD_HYBRID_LAYERS];
        strd_hybrid_layout(L, type);
        int red[STRD_HYBRID_LAYERS], nred = 0, want = extra;
        for (int l = 1; l < L; ++l) {
            if (type[l] == STRD_LAYER_ATTN) { red[nred++] = l; want = extra; }
            else if (type[l] == STRD_LAYER_MAMBA && want > 0) { red[nred++] = l; --want; }
        }
        int last = 0;
        while (last + 1 < nred && red[last + 1] <= 33) ++last;
        for (int l = 0; l < L; ++l) alpha_out[l] = 1.0;
        for (int i = 0; i < nred; ++i) {
            const double a = i >= last ? 0.15 : 0.32 + (0.15 - 0.32) * (double)i / (double)last;
            for (int l = red[i]; l < L; ++l) alpha_out[l] = a;
        }
        return STRD_OK;
    }
    return STRD_EINVAL;
}

}  // extern "C"
