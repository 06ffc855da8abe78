/*
 * strd.h -- C ABI of the stateful token-reduced prefill library for MI355X (gfx950).
 *
 * One hybrid layer of "Stateful Token Reduction for Long-Video Hybrid VLMs" is
 * prefilled on a reduced token set: score the vision tokens against the text
 * query, keep the top K in temporal order, compact every per-token tensor, run the
 * layer mixer (Mamba-2 scan or causal GQA attention) on the K + M survivors.
 *
 * Common rules for every entry point
 *   - A sequence is N vision tokens followed by M text tokens (Sec. 3.1).  All
 *     tensors are token-major, contiguous, batch 1.
 *   - Pointers marked [dev] are device pointers owned by the caller; [host] are
 *     host pointers.  The library allocates, frees and retains no device memory, with
 *     one exception that is stated where it applies: strd_linear hands the products its
 *     own kernel is not built for to rocBLAS and keeps that library's handle (and whatever
 *     it allocates) for the life of the process.
 *   - `io` is the element type of the tensors declared `const void*` / `void*`
 *     (STRD_F32 or STRD_BF16); accumulation, exponentials, decay, state and scores
 *     are always fp32.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and the call returns without synchronising.
 *   - `ws` is caller-provided scratch [dev] of at least the size the matching
 *     *_workspace() query returns (may be NULL when that size is 0); its contents
 *     are undefined before and after the call.  Tensor buffers and `ws` must be 16-byte
 *     aligned (the matrix-core kernels move 16-byte vectors straight from the caller's
 *     pointers; a misaligned buffer on such a shape is STRD_EINVAL), fp32 vectors of
 *     per-head or per-token scalars (A, D, dt) need only their natural alignment.
 *   - Return value: STRD_OK or a negative strd_status.  On STRD_EINVAL,
 *     STRD_EUNSUPPORTED and STRD_EWORKSPACE nothing was launched and no output was
 *     written.  STRD_EHIP reports a failed launch (hipGetLastError).
 *   - Shapes the kernels are not built for give STRD_EUNSUPPORTED; there is no CPU
 *     or library fallback.
 *   - The two scores and the two mixers each have two device kernels: a matrix-core
 *     (MFMA) kernel for bf16 tensors in the tile shapes listed at strd_*_kernel_path
 *     below, and a plain SIMT kernel in fp32 arithmetic that serves fp32 tensors (whose
 *     1e-4 tolerance bf16 matrix cores cannot meet) and every other bf16 shape.  The SIMT
 *     kernels are one to two orders of magnitude slower; which one a call will run is
 *     never implicit: strd_*_kernel_path answers it from the shape alone.
 */
#ifndef STRD_H
#define STRD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { STRD_F32 = 0, STRD_BF16 = 1 } strd_dtype;

typedef enum {
    STRD_OK = 0,
    STRD_EINVAL = -1,       /* inconsistent sizes or NULL where data is required  */
    STRD_EUNSUPPORTED = -2, /* valid problem, no kernel built for this shape       */
    STRD_EWORKSPACE = -3,   /* ws == NULL or ws_bytes too small                    */
    STRD_EHIP = -4          /* the HIP runtime refused a launch                    */
} strd_status;

/* Human-readable name of a status code (static storage, never NULL). */
const char *strd_status_string(int status);

/* ABI version: major * 1000 + minor. */
int strd_version(void);

/* Measurement aid (used by the benchmark, not by the path; for callers that want to know what
 * the matrix cores of their chip sustain): `workgroups` x 4 waves each issue `iters` x 32
 * independent v_mfma_f32_32x32x16_bf16 products on register-resident operands and write one
 * float per thread to out [dev] [workgroups * 256] (a checksum, so that nothing is optimised
 * away).  `mode` bit 0: random bf16 operands in +-[1, 2) instead of 1.0 everywhere; bit 1: the
 * 16 x 16 x 32 form of the instruction, twice as many products of half the size.  One launch is
 * workgroups * 4 * iters * 32 * 32768 flop in either form; time it with events on `stream`.
 * STRD_EINVAL for out == NULL, workgroups < 1, iters < 1 or mode outside 0..3. */
int strd_mfma_rate_probe(float *out, int workgroups, int iters, int mode, void *stream);

/* Which device kernel a call with these sizes runs: STRD_PATH_MFMA (bf16 matrix cores),
 * STRD_PATH_SIMT (fp32 arithmetic on the vector units: fp32 tensors, and bf16 shapes outside
 * the matrix-core tiles) or STRD_PATH_NONE (the call would return STRD_EINVAL or
 * STRD_EUNSUPPORTED).  Matrix-core shapes, all bf16: score_attn and attn_prefill d in {64, 128};
 * score_mamba n in {64, 128}; ssd_prefill n in {64, 128} and P a multiple of 32 (and every
 * tensor below 4 GiB).  Host-only, touches no device. */
typedef enum { STRD_PATH_NONE = 0, STRD_PATH_MFMA = 1, STRD_PATH_SIMT = 2 } strd_kernel_path;
int strd_score_attn_kernel_path(int M, int N, int Hq, int Hkv, int d, strd_dtype io);
int strd_score_mamba_kernel_path(int M, int N, int H, int G, int n, strd_dtype io);
int strd_ssd_prefill_kernel_path(int T, int H, int P, int G, int n, strd_dtype io);
int strd_attn_prefill_kernel_path(int T, int Hq, int Hkv, int d, strd_dtype io);

/* ---------------------------------------------------------------------------
 * score_attn -- attention-layer importance (Sec. 3.1 "Attention Layers"):
 *     s_i = 1/(M*Hq) * sum_{m,h} softmax_i( scale * q_m^h . k_i^{kv(h)} )
 * The softmax runs over the N vision keys only, so sum_i s_i = 1.  Query head h
 * reads key head kv(h) = h / (Hq/Hkv).
 *   q_txt  [dev] [M, Hq, d]   text-row queries (already projected / rotated)
 *   k_vis  [dev] [N, Hkv, d]  vision-row keys
 *   scores [dev] [N] fp32     output
 * Requires M,N >= 1, Hq % Hkv == 0, scale > 0.  Deterministic (fixed reduction order).
 * ------------------------------------------------------------------------- */
size_t strd_score_attn_workspace(int M, int N, int Hq, int Hkv, int d, strd_dtype io);
int strd_score_attn(const void *q_txt, const void *k_vis, float *scores, int M, int N, int Hq,
                    int Hkv, int d, float scale, strd_dtype io, void *ws, size_t ws_bytes,
                    void *stream);

/* ---------------------------------------------------------------------------
 * score_mamba -- Decoupled Content Alignment (Eq. "ssm_importance"), the
 * decay-free Mamba-2 score.  Delta is per head while b, c are per group, so the
 * mean runs over every head:
 *     s_i = 1/(M*H) * sum_{m,h} dt_i^h * | b_i^{g(h)} . c_m^{g(h)} |,  g(h) = h/(H/G)
 * which equals the paper's group form with the group-mean of Delta in b-bar.
 *   B_vis  [dev] [N, G, n]   vision-row input projections b
 *   C_txt  [dev] [M, G, n]   text-row output projections c
 *   dt_vis [dev] [N, H] fp32 discretisation steps (> 0, already softplus'd)
 *   scores [dev] [N] fp32    output
 * Requires M,N >= 1, H % G == 0.  Deterministic.
 * ------------------------------------------------------------------------- */
size_t strd_score_mamba_workspace(int M, int N, int H, int G, int n, strd_dtype io);
int strd_score_mamba(const void *B_vis, const void *C_txt, const float *dt_vis, float *scores,
                     int M, int N, int H, int G, int n, strd_dtype io, void *ws, size_t ws_bytes,
                     void *stream);

/* ---------------------------------------------------------------------------
 * score_mamba_full -- the Full Mamba Dynamic score (|w_{t,j}| of Eq. "ssm_weight"),
 * which the decay-free score above is ablated against: every term carries the
 * decay of the recurrence from vision token i to text row m,
 *     s_i = 1/(M*H) * sum_{m,h} dt_i^h * | b_i^{g(h)} . c_m^{g(h)} | * prod_{u=i+1}^{N+m} exp(dt_u^h * A^h).
 * With A = 0 it equals score_mamba.
 *   B_vis  [dev] [N, G, n]      C_txt [dev] [M, G, n]
 *   dt_all [dev] [N+M, H] fp32  steps of every token, vision rows first (the decay runs through
 *                               the later vision tokens and the text rows up to m)
 *   A      [dev] [H] fp32 (< 0) scores [dev] [N] fp32 output
 * Requires M,N >= 1, H % G == 0; the workspace is always needed.  Deterministic.
 * ------------------------------------------------------------------------- */
size_t strd_score_mamba_full_workspace(int M, int N, int H, int G, int n, strd_dtype io);
int strd_score_mamba_full(const void *B_vis, const void *C_txt, const float *dt_all, const float *A,
                          float *scores, int M, int N, int H, int G, int n, strd_dtype io, void *ws,
                          size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * select_topk -- keep the K highest-scoring vision tokens, in temporal order
 * (Sec. 3.1 "Token Selection").  Ties at the K-th score go to the lowest index.
 *   scores [dev] [N] fp32, finite and >= 0 (both score kinds are); -0.0 counts as 0.  Other
 *          values do not break the call: negative scores and infinities order as numbers, NaNs
 *          by their bit patterns (positive-signed above +inf, negative-signed below -inf), and
 *          exactly K indices are written in every case
 *   idx    [dev] [K] int32 output, strictly ascending
 * Requires 1 <= K <= N.  Bit-exact and deterministic.
 *   ws     [dev] strd_select_topk_workspace(N, K) bytes (0 up to 32768 scores and above 2^20;
 *          about 26 KB of histograms and counters between); contents need not be initialised and
 *          are not preserved; STRD_EWORKSPACE if it is missing or too small
 * ------------------------------------------------------------------------- */
size_t strd_select_topk_workspace(int N, int K);
int strd_select_topk(const float *scores, int N, int K, int32_t *idx, void *ws, size_t ws_bytes,
                     void *stream);

/* select_topk_noalloc -- strd_select_topk for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result,
 * bit for bit; no workspace argument: the histograms and counters of the selection live in a
 * 26 KB array inside the library's image, one copy per GPU, held until the process ends.  The
 * call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine).
 *   N at most strd_select_topk_noalloc_max_n() = 1 048 576 scores; more gives STRD_EUNSUPPORTED
 *   and nothing is launched.  Other arguments and errors as strd_select_topk.
 * All calls on one GPU share that GPU's array (every call clears what it needs on `stream`
 * before using it, so nothing is carried from one call to the next): calls that overlap on one
 * GPU -- different streams, or different threads -- race; serialise them.  The first call on each
 * GPU looks the array's device address up (hipGetSymbolAddress); make that first call outside
 * any stream capture. */
int strd_select_topk_noalloc_max_n(void);
int strd_select_topk_noalloc(const float *scores, int N, int K, int32_t *idx, void *stream);

/* ---------------------------------------------------------------------------
 * compact -- drop the unselected vision tokens of one per-token tensor
 * (Sec. 3.1: retained tokens continue; text tokens are never dropped):
 *     dst[r, :]   = src[idx[r], :]   r < K
 *     dst[K+m, :] = src[N+m, :]      m < M
 *     pos_out     = the same gather applied to pos_in (identity map if pos_in NULL)
 *   src     [dev] [N+M rows of row_bytes]      dst [dev] [K+M rows]; must not overlap src
 *   idx     [dev] [K] int32, ascending, each in [0, N) (not checked on the device)
 *   pos_in  [dev] [N+M] int32 or NULL          pos_out [dev] [K+M] int32 or NULL
 * row_bytes > 0 and a multiple of 4; rows need only their natural alignment when
 * row_bytes % 16 != 0.  src/dst may be NULL when only the position map is wanted.
 * Requires 0 <= K <= N, M >= 0.  Bit-exact copy.
 * ------------------------------------------------------------------------- */
int strd_compact(const void *src, const int32_t *idx, void *dst, int N, int M, int K,
                 int64_t row_bytes, const int32_t *pos_in, int32_t *pos_out, void *stream);

/* compact_batch -- the same gather for up to STRD_COMPACT_MAX tensors that share one index
 * list (a reducing layer compacts every mixer input and the hidden states), in one launch.
 *   items [host] [n_items] {src [dev], dst [dev], row_bytes}; read before the call returns
 * Every item obeys the rules of strd_compact; n_items may be 0 when only pos_out is wanted. */
#define STRD_COMPACT_MAX 8
typedef struct {
    const void *src;
    void *dst;
    int64_t row_bytes;
} strd_compact_item;
int strd_compact_batch(const strd_compact_item *items, int n_items, const int32_t *idx, int N, int M,
                       int K, const int32_t *pos_in, int32_t *pos_out, void *stream);

/* ---------------------------------------------------------------------------
 * Packed batches of sequences -- scoring, selection and compaction (Sec. 3.1,
 * "Layer-wise Token Importance" and the token selection after it) for several
 * sequences of different lengths in one set of launches.  Each sequence is
 * reduced on its own, exactly as by the single-sequence calls above; the
 * point is that short sequences, whose calls are bound by launch latency,
 * share their launches.
 *
 * Layout.  The per-token tensors of the sequences lie one after the other
 * along the token axis (no padding): sequence b is rows
 * [row0_b, row0_b + N_b + M_b), row0_b = sum over earlier sequences of
 * (N + M), its N_b vision rows first, then its M_b text rows.  `seqs` is a
 * HOST array of `nseq` descriptors, read before the call returns.
 *   scores  [dev] [nseq, ld] fp32: row b holds the N_b scores of sequence b
 *           (entries past N_b are not touched); ld >= every N_b, ld % 4 == 0.
 *   idx     [dev] [sum of K_b] int32: the kept vision tokens of sequence b,
 *           ascending and local to the sequence (0 .. N_b - 1), start at
 *           offset sum of earlier K.
 *   compacted tensors: sequence b is rows [o_b, o_b + K_b + M_b),
 *           o_b = sum over earlier sequences of (K + M).
 *   pos_out [dev] [sum of (K_b + M_b)] int32: row number inside its own
 *           sequence's N_b + M_b input rows (pos_in == NULL), or
 *           pos_in[row0_b + that row]; pos_in [dev] [sum of (N_b + M_b)].
 * Requires 1 <= nseq <= STRD_VARLEN_MAX, every N_b >= 1, M_b >= 1,
 * 1 <= K_b <= N_b (the scores ignore K_b; select and compact use it), and for
 * strd_select_topk_varlen every N_b <= strd_select_topk_varlen_max_n()
 * (32768: one workgroup per sequence), else STRD_EINVAL / STRD_EUNSUPPORTED.
 * The same alignment rules as the single-sequence calls apply to the packed
 * base pointers.  Tie-breaking, NaN handling and error behaviour are those of
 * the single-sequence calls.
 * ------------------------------------------------------------------------- */
#define STRD_VARLEN_MAX 64
typedef struct strd_seq {
    int32_t N; /* vision tokens */
    int32_t M; /* text tokens (they follow the vision tokens) */
    int32_t K; /* vision tokens to keep */
} strd_seq;
size_t strd_score_attn_varlen_workspace(const strd_seq *seqs, int nseq, int Hq, int Hkv, int d, strd_dtype io);
int strd_score_attn_varlen(const void *q_all /* [dev] [rows, Hq, d] */, const void *k_all /* [dev] [rows, Hkv, d] */,
                           float *scores, int ld, const strd_seq *seqs, int nseq, int Hq, int Hkv, int d,
                           float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream);
size_t strd_score_mamba_varlen_workspace(const strd_seq *seqs, int nseq, int H, int G, int n, strd_dtype io);
int strd_score_mamba_varlen(const void *B_all /* [dev] [rows, G, n] */, const void *C_all /* [dev] [rows, G, n] */,
                            const float *dt_all /* [dev] [rows, H] */, float *scores, int ld,
                            const strd_seq *seqs, int nseq, int H, int G, int n, strd_dtype io, void *ws,
                            size_t ws_bytes, void *stream);
int strd_select_topk_varlen_max_n(void);
int strd_select_topk_varlen(const float *scores, int ld, const strd_seq *seqs, int nseq, int32_t *idx,
                            void *stream);
int strd_compact_varlen(const strd_compact_item *items, int n_items, const int32_t *idx, const strd_seq *seqs,
                        int nseq, const int32_t *pos_in, int32_t *pos_out, void *stream);

/* ---------------------------------------------------------------------------
 * ssd_prefill -- Mamba-2 mixer over T tokens (Eqs. "ssm_state_update",
 * "ssm_output"), per head h with group g(h):
 *     S_t = exp(dt_t * A) * S_{t-1} + x_t (dt_t * b_t)^T ,   y_t = S_t c_t (+ D x_t)
 * evaluated in its chunked (state-space-dual) form with the state carried on chip.
 *   x   [dev] [T, H, P]          dt [dev] [T, H] fp32 (> 0)     A [dev] [H] fp32 (<= 0)
 *   B,C [dev] [T, G, n]          D  [dev] [H] fp32 or NULL
 *   S_in  [dev] [H, P, n] fp32 or NULL (zero state)
 *   y     [dev] [T, H, P]        S_out [dev] [H, P, n] fp32 or NULL
 * The bf16 matrix-core kernels add D x_t inside the token product (D joins the bf16 weight of
 * token t on itself), i.e. that term carries a relative rounding error of up to 2^-9, like every
 * other term of the sum and like the bf16 output itself.
 * `chunk` is the chunk length of the caller's formulation (> 0).  It is validated and
 * otherwise unused: it does NOT select the tiling.  The kernels always cut time into
 * 64-token steps and carry the state across them on chip, so results do not depend on
 * `chunk` at all.  S_out of one call fed as S_in of the next continues the same scan.
 *   ws  [dev] strd_ssd_prefill_workspace(T, ...) bytes: 0 for short sequences; for long ones the
 *       sequence is cut into segments that run side by side, and the local end state and total
 *       decay of every segment but the last pass through the workspace ((segments - 1) * H * P * n
 *       + segments * H floats).  Too small or NULL when needed: STRD_EWORKSPACE.
 * Requires T >= 0, H % G == 0.
 * ------------------------------------------------------------------------- */
size_t strd_ssd_prefill_workspace(int T, int H, int P, int G, int n, int chunk, strd_dtype io);
int strd_ssd_prefill(const void *x, const float *dt, const float *A, const void *B, const void *C,
                     const float *D, const float *S_in, void *y, float *S_out, int T, int H, int P,
                     int G, int n, int chunk, strd_dtype io, void *ws, size_t ws_bytes,
                     void *stream);

/* ssd_prefill_gather -- ssd_prefill on the K + M surviving tokens WITHOUT a compacted copy of
 * the mixer inputs: token t of the scan is row idx[t] (t < K) or N + (t - K) of the
 * uncompacted x, dt, B, C (N + M rows each).  Equal, bit for bit, to compacting the four
 * tensors with strd_compact and calling strd_ssd_prefill, minus that HBM round trip.
 *   idx [dev] [K] int32, ascending, each in [0, N)     y [dev] [K+M, H, P] (dense)
 *   ws  [dev] strd_ssd_prefill_workspace(K + M, ...) bytes, as for the dense call on K + M tokens.
 * Only shapes the matrix-core kernels cover (bf16, n in {64, 128}, P % 32 == 0, K + M >= 1);
 * anything else gives STRD_EUNSUPPORTED (compact, then call strd_ssd_prefill). */
int strd_ssd_prefill_gather(const void *x, const float *dt, const float *A, const void *B, const void *C,
                            const float *D, const float *S_in, const int32_t *idx, void *y, float *S_out,
                            int N, int M, int K, int H, int P, int G, int n, int chunk, strd_dtype io,
                            void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * attn_prefill -- causal softmax attention with grouped-query heads over T tokens
 * (App. "Attention via Kernel Functions", first equation):
 *     o_t^h = sum_{j<=t} softmax_j( scale * q_t^h . k_j^{kv(h)} ) v_j^{kv(h)}
 * in the order the tokens have in the (compacted) sequence.
 *   q [dev] [T, Hq, d]    k, v [dev] [T, Hkv, d]    o [dev] [T, Hq, d]
 * Requires T >= 0, Hq % Hkv == 0, scale > 0 (else STRD_EINVAL).
 * ------------------------------------------------------------------------- */
size_t strd_attn_prefill_workspace(int T, int Hq, int Hkv, int d, strd_dtype io);
int strd_attn_prefill(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv,
                      int d, float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Block glue around the mixers: what a hybrid layer does between
 * its projections and the scan or attention, apart from matrix products.  The paper builds on
 * the Mamba-2 block and does not restate these operations; they follow that block's published
 * definition.  All: [dev] tensors of the io dtype (weights included) unless stated, fp32
 * arithmetic, one rounding on output, asynchronous on `stream`, T = 0 allowed.
 *
 * rmsnorm:        out[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + eps) * w            x, out [T, d], w [d]
 * gated_rmsnorm:  v = y * silu(z); out = v / sqrt(mean_group(v^2) + eps) * w    y, out [T, D]; z rows of
 *                 pitch ldz >= D elements; `groups` equal groups of D / groups channels each; w [D]
 * conv1d_silu:    causal depthwise convolution over tokens with zero history, then SiLU,
 *                   o[t,c] = silu(b[c] + sum_{k<W} w[c,k] * xbc[t-(W-1)+k, c]),
 *                 on the first Cx + 2*Cb columns of xbc (rows of pitch ld elements); columns
 *                 [0,Cx) go to x_out [T,Cx], the next Cb to B_out [T,Cb], the last Cb to C_out
 *                 [T,Cb]; w [Cx+2*Cb, W], b [Cx+2*Cb] or NULL.  Cx, Cb, ld multiples of 8 and
 *                 16-byte (bf16) / 32-byte (fp32) aligned bases, W <= 4, else STRD_EUNSUPPORTED.
 * softplus_dt:    dt[t,h] = log(1 + exp(raw[t, col0+h] + bias[h])), raw rows of pitch ld in the io
 *                 dtype, bias [H] fp32 or NULL, dt [T,H] fp32.
 * linear:         out[T,Nd] = x[T,Kd] . w[Kd,Nd] (+ residual[T,Nd], which may be `out` itself): the
 *                 projections of a block, fp32 accumulation, the residual added in fp32 before the one
 *                 rounding.  Large bf16 products (see linear_mfma; at least one 256 x 256 output tile per
 *                 CU, 16-byte aligned pointers) run on the library's own kernel; everything else (fp32,
 *                 other shapes, small products) is handed to rocBLAS.  That second path is the one place
 *                 where something is retained: its first use in a process creates a rocBLAS handle (which
 *                 allocates device workspace of its own) and keeps it until the process ends; calls are
 *                 serialised on it.  Callers that must not allocate use strd_linear_mfma.
 * linear_library: the same product by rocBLAS whatever the shape (what strd_linear falls back to; kept as an
 *                 entry point so that the two can be timed side by side).
 * linear_mfma:    the same product by the library's own kernel only (bf16 matrix cores): no handle, no
 *                 allocation, nothing kept between calls.  bf16, Kd a multiple of 64, Nd a multiple of 8,
 *                 x and w below 4 GiB each, all pointers 16-byte aligned (STRD_EINVAL if not); other shapes
 *                 return STRD_EUNSUPPORTED (strd_linear_mfma_supported answers that from the shape alone:
 *                 1 or 0).  `residual` may be `out`.  Any size is computed correctly; below one output tile
 *                 per CU most of the chip idles.
 * ------------------------------------------------------------------------- */
int strd_linear(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd,
                strd_dtype io, void *stream);
int strd_linear_mfma(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd,
                     strd_dtype io, void *stream);
int strd_linear_library(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd,
                        strd_dtype io, void *stream);
int strd_linear_mfma_supported(int T, int Kd, int Nd, strd_dtype io);
int strd_rmsnorm(const void *x, const void *w, void *out, int T, int d, float eps, strd_dtype io, void *stream);
int strd_gated_rmsnorm(const void *y, const void *z, int ldz, const void *w, void *out, int T, int D,
                       int groups, float eps, strd_dtype io, void *stream);
int strd_conv1d_silu(const void *xbc, int ld, const void *w, const void *b, void *x_out, void *B_out,
                     void *C_out, int T, int Cx, int Cb, int W, strd_dtype io, void *stream);
int strd_softplus_dt(const void *raw, int ld, int col0, const float *bias, float *dt, int T, int H,
                     strd_dtype io, void *stream);

/* ---------------------------------------------------------------------------
 * Variants around the reduced prefill.
 *
 * avgpool -- the average-pooling reduction that the "Reduction Types" ablation (Sec. 4,
 * ablation table, right half) sets against query-based selection.  The paper does not state
 * the window shape; here the N vision rows are cut into K consecutive windows
 * [floor(j N / K), floor((j+1) N / K)), j < K, each replaced by its mean (fp32 accumulation in
 * row order, one rounding), and the M text rows follow unchanged.  src [dev] [N+M, D], dst [dev]
 * [K+M, D], both of dtype io and contiguous (src == dst == NULL: positions only); pos_out [dev]
 * [K+M] or NULL receives pos_in (NULL = identity) of the first row of each window, then of the
 * text rows.  1 <= K <= N (K = 0 only with N = 0).
 *
 * ssd_decode_step -- one token of the Mamba-2 recurrence (Eqs. ssm_state_update, ssm_output with
 * T = 1) from the state a prefill left in S_out:  S <- exp(dt_h A_h) S + dt_h x b^T (in place),
 * y = S c + D x.  x, y [dev] [H, P] and B, C [dev] [G, n] of dtype io; dt, A, D (or NULL) [dev]
 * fp32 [H]; S [dev] fp32 [H, P, n], read and written.
 *
 * attn_decode_step -- the newest token's causal attention over a cache of T key/value rows, its
 * own row included (the last row of the appendix's softmax-attention equation): q, o [dev]
 * [Hq, d]; k_cache, v_cache [dev] [T, Hkv, d] -- after a reduced prefill these are the K + M
 * surviving rows followed by the generated ones.  d in {64, 128}, Hq / Hkv in {1, 2, 4, 8},
 * 16-byte (bf16) / 32-byte (fp32) aligned bases, else STRD_EUNSUPPORTED; scale > 0.  Workspace
 * [dev]: strd_attn_decode_step_workspace bytes, 16-byte aligned (STRD_EWORKSPACE otherwise).
 *
 * All asynchronous on `stream`; no call allocates.
 * ------------------------------------------------------------------------- */
int strd_avgpool(const void *src, void *dst, int N, int M, int K, int D, strd_dtype io, const int32_t *pos_in,
                 int32_t *pos_out, void *stream);
int strd_ssd_decode_step(const void *x, const float *dt, const float *A, const void *B, const void *C,
                         const float *D, float *S, void *y, int H, int P, int G, int n, strd_dtype io,
                         void *stream);
size_t strd_attn_decode_step_workspace(int T, int Hq, int Hkv, int d, strd_dtype io);
int strd_attn_decode_step(const void *q, const void *k_cache, const void *v_cache, void *o, int T, int Hq,
                          int Hkv, int d, float scale, strd_dtype io, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * schedule_budgets -- per-layer token budgets of a retention schedule (Sec. 3.2
 * and App. "Reduction Schedule Configurations").  alpha_l is relative to the
 * original count N0; budgets never grow with depth and never fall below
 * min(K_min, current count):
 *     K_l = min(K_{l-1}, max(floor(alpha_l * N0), min(K_min, K_{l-1}))),  K_{-1} = N0
 *   alpha [host] [L] doubles in [0, 1]      K_out [host] [L] int32
 * Host-only helper; touches no device.
 * ------------------------------------------------------------------------- */
int strd_schedule_budgets(const double *alpha, int L, int N0, int K_min, int32_t *K_out);

/* Sigmoid retention schedule (App. "Sigmoid Schedule"), layers l = 0..L-1:
 *     alpha_l = a_end + (a_start - a_end) * sigmoid(k * (x0 - l / L))
 *   alpha_out [host] [L] doubles */
int strd_schedule_sigmoid(int L, double a_start, double a_end, double k, double x0,
                          double *alpha_out);

/* Step-decay retention schedule (App. "Step Decay Schedule"): alpha_l = alpha[r] for the layers
 * lo[r]..hi[r] (inclusive, 0-indexed; later ranges win), 1.0 elsewhere.
 *   lo, hi [host] [nranges] ints   alpha [host] [nranges] doubles in [0,1]   alpha_out [host] [L] */
int strd_schedule_step_decay(const int *lo, const int *hi, const double *alpha, int nranges, int L,
                             double *alpha_out);

/* Layer types of the 62-layer hybrid the schedules of the paper are written for (App. "Reduction
 * Schedule Configurations"): attention at layers 7, 16, 25, 34, 43, 52; the other 56 layers
 * alternate Mamba-2, MLP starting with Mamba-2 (28 + 28; the paper gives the counts, not the order).
 *   type_out [host] [L] int32 of STRD_LAYER_*; a shorter or longer L follows the same rule. */
enum { STRD_LAYER_MAMBA = 0, STRD_LAYER_MLP = 1, STRD_LAYER_ATTN = 2, STRD_HYBRID_LAYERS = 62 };
int strd_hybrid_layout(int L, int32_t *type_out);

/* The named schedules of the same table, as retention ratios for the STRD_HYBRID_LAYERS layers:
 * "attn_only_1st_attn", "all_attn_25", "all_attn_35", "all_attn_50", "first_mamba",
 * "second_mamba" (ranges as printed), "sigmoid_25", "sigmoid_35", "sigmoid_50" (k = 20, x0 = 0.11 /
 * 0.24 / 0.41, 1.0 -> 0.125), "all_attn_1m", "all_attn_2m" (the table only says 0.32 -> 0.15 over
 * the 6 attention layers plus 1 or 2 Mamba layers before each: taken as a linear fall over the
 * reducing layers up to layer 33, held afterwards).  Unknown name: STRD_EINVAL.
 *   alpha_out [host] [STRD_HYBRID_LAYERS] doubles */
int strd_schedule_named(const char *name, double *alpha_out);

#ifdef __cplusplus
}
#endif
#endif /* STRD_H */
