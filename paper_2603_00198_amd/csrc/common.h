// Shared device/host helpers for the strd kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "strd.h"

namespace strd {

typedef __bf16 bf16_t;

constexpr int kWave = 64;   // CDNA wavefront width
constexpr int kXcd = 8;     // MI355X: 8 XCDs, workgroups are dealt to them round-robin

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return static_cast<float>(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return static_cast<bf16_t>(v); }

__host__ __device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ __forceinline__ size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Deal consecutive logical units to the same XCD: hardware sends workgroup b to XCD b % 8,
// so unit = (b % 8) * ceil(n / 8) + b / 8 keeps neighbours (which share operands) on one L2.
// Returns n or more for the padding workgroups of the last column; callers skip those.
__device__ __forceinline__ int xcd_swizzle(int b, int n) {
    const int per = (n + kXcd - 1) / kXcd;
    return (b % kXcd) * per + b / kXcd;
}
__host__ __forceinline__ int xcd_grid(int n) { return (n + kXcd - 1) / kXcd * kXcd; }

// ---- packed batches of sequences (the *_varlen entry points) ---------------------------------
// The per-token tensors of several sequences lie one after the other along the token axis:
// sequence b is rows [row0[b], row0[b] + N[b] + M[b]), vision rows first.  The table travels in
// the kernel arguments; a kernel instantiated with OneSeq takes its tensors as one sequence.
constexpr int kMaxSeqs = STRD_VARLEN_MAX;
struct OneSeq {};
struct SeqTab {
    int row0[kMaxSeqs], N[kMaxSeqs], M[kMaxSeqs], K[kMaxSeqs];
    int koff[kMaxSeqs];  // retained vision tokens of the sequences before b (offset into the index list)
    int ooff[kMaxSeqs];  // rows of the compacted tensors before b
};
template <class SEQ> constexpr bool is_varlen() { return std::is_same<SEQ, SeqTab>::value; }

// ---- asynchronous global -> LDS tile copy (no VGPR staging) ---------------------------------
// A tile is ROWS rows of VR 16-byte vectors, stored in LDS with PAD pad vectors per row (pitch
// VR + PAD vectors, which keeps 16-byte row reads and transposing reads off each other's banks).
// global_load_lds writes lane l of a wave to (uniform LDS base) + 16 * l, so the tile is filled
// slot by slot: slot s = row * (VR + PAD) + cv; pad slots (cv >= VR) re-read the row's last vector.
// Slots are dealt to the NW waves of the workgroup 64 at a time; lanes whose slot lies past the
// end of the tile copy nothing, so the tile occupies exactly ROWS * (VR + PAD) * 16 bytes.
// SKIP_PAD: lanes on pad slots copy nothing either (the pad bytes stay unwritten and must never
// be read into a result), which saves PAD / (VR + PAD) of the copy traffic.
template <int ROWS, int VR, int NW, int PAD = 1, bool SKIP_PAD = false>
struct AsyncTile {
    static constexpr int kVP = VR + PAD;                                // vectors per LDS row
    static constexpr int kPitch = kVP * 8;                              // bf16 elements per LDS row
    static constexpr int kSlots = ROWS * kVP;
    static constexpr int kIssues = (kSlots + 64 * NW - 1) / (64 * NW);  // instructions per wave
    static constexpr int kBytes = kSlots * 16;

    // Row and vector of the slot this lane fills with its i-th instruction.
    __device__ static __forceinline__ void slot(int wave, int lane, int i, int &row, int &cv) {
        const int s = (i * NW + wave) * 64 + lane;
        row = min(s / kVP, ROWS - 1);
        cv = min(s % kVP, VR - 1);
    }
    // Issue this lane's i-th copy: 16 bytes from `src` to its slot of the tile at `lds_tile`.
    __device__ static __forceinline__ void issue(const void *src, void *lds_tile, int wave, int i) {
        char *dst = reinterpret_cast<char *>(lds_tile) + (i * NW + wave) * 1024;
        const int s = (i * NW + wave) * 64 + (int)(threadIdx.x & 63);
        if (((i + 1) * NW * 64 <= kSlots || s < kSlots) &&  // only the last round can run past the tile
            (!SKIP_PAD || s % kVP < VR))
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    }
};
// Wait until every copy this wave issued has landed (call before the barrier that publishes).
__device__ __forceinline__ void async_tile_wait() { __builtin_amdgcn_s_waitcnt(0); }

// ---- transposing LDS reads (ds_read_b64_tr_b16) ----------------------------------------------
// Within each group of 16 lanes, lane r passes the address of element [k0 + r/4][c0 + 4*(r%4)] of
// a row-major bf16 tile and receives [k0..k0+3][c0 + r]: four consecutive rows of one column,
// which is what an MFMA operand needs when the contraction index runs along the tile's rows.
// The reads are issued from inline assembly, eight at a time with one wait: the compiler's own
// builtin carries no memory operand, so every use of it would wait for all outstanding
// asynchronous global -> LDS copies and serialise the prefetch.
typedef short strd_s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 strd_bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 strd_bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t lds_offset(const void *p) {
    return (uint32_t)(size_t)(__attribute__((address_space(3))) const char *)p;
}

// r[i] = transposed read at byte offset Oi from p.
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ void lds_read_tr8(const void *p, strd_s16x4 (&r)[8]) {
    const uint32_t a = lds_offset(p);
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8 offset:%9\n\t"
        "ds_read_b64_tr_b16 %1, %8 offset:%10\n\t"
        "ds_read_b64_tr_b16 %2, %8 offset:%11\n\t"
        "ds_read_b64_tr_b16 %3, %8 offset:%12\n\t"
        "ds_read_b64_tr_b16 %4, %8 offset:%13\n\t"
        "ds_read_b64_tr_b16 %5, %8 offset:%14\n\t"
        "ds_read_b64_tr_b16 %6, %8 offset:%15\n\t"
        "ds_read_b64_tr_b16 %7, %8 offset:%16\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
        : "v"(a), "i"(O0), "i"(O1), "i"(O2), "i"(O3), "i"(O4), "i"(O5), "i"(O6), "i"(O7)
        : "memory");
}
// The same eight reads without the wait: the results may be used only after lds_settle8() on
// the same registers.  Splitting issue and wait lets a wave put all the LDS reads of a step in
// flight at once instead of paying one LDS round trip per group of reads.  Between the two the
// compiler takes the registers for loaded, so it must never have a reason to move them: a kernel
// that uses this has to fit its register budget without spilling (the build is checked for it).
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ void lds_issue_tr8(const void *p, strd_s16x4 (&r)[8]) {
    const uint32_t a = lds_offset(p);
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8 offset:%9\n\t"
        "ds_read_b64_tr_b16 %1, %8 offset:%10\n\t"
        "ds_read_b64_tr_b16 %2, %8 offset:%11\n\t"
        "ds_read_b64_tr_b16 %3, %8 offset:%12\n\t"
        "ds_read_b64_tr_b16 %4, %8 offset:%13\n\t"
        "ds_read_b64_tr_b16 %5, %8 offset:%14\n\t"
        "ds_read_b64_tr_b16 %6, %8 offset:%15\n\t"
        "ds_read_b64_tr_b16 %7, %8 offset:%16"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
        : "v"(a), "i"(O0), "i"(O1), "i"(O2), "i"(O3), "i"(O4), "i"(O5), "i"(O6), "i"(O7)
        : "memory");
}
// Four reads, same contract as lds_issue_tr8 / lds_settle8.
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void lds_issue_tr4(const void *p, strd_s16x4 (&r)[4]) {
    const uint32_t a = lds_offset(p);
    asm volatile(
        "ds_read_b64_tr_b16 %0, %4 offset:%5\n\t"
        "ds_read_b64_tr_b16 %1, %4 offset:%6\n\t"
        "ds_read_b64_tr_b16 %2, %4 offset:%7\n\t"
        "ds_read_b64_tr_b16 %3, %4 offset:%8"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(a), "i"(O0), "i"(O1), "i"(O2), "i"(O3)
        : "memory");
}
__device__ __forceinline__ void lds_settle4(strd_s16x4 (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : : "memory");
}
// Wait for every LDS operation of the wave; the registers pass through the statement so that no
// use of them can be scheduled before it.
__device__ __forceinline__ void lds_settle8(strd_s16x4 (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 :
                 : "memory");
}
// The same with up to N later LDS operations of the wave still outstanding (they return in order).
template <int N>
__device__ __forceinline__ void lds_settle8_but(strd_s16x4 (&r)[8]) {
    static_assert(N >= 0 && N < 16, "lgkmcnt has 4 bits");
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 : "i"(N)
                 : "memory");
}
__device__ __forceinline__ strd_bf16x8 tr_pair(strd_s16x4 lo, strd_s16x4 hi) {
    return __builtin_shufflevector(__builtin_bit_cast(strd_bf16x4, lo), __builtin_bit_cast(strd_bf16x4, hi), 0, 1, 2, 3,
                                   4, 5, 6, 7);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory,
// which on gfx9 means waiting for every outstanding vector-memory operation of the wave -- all
// the asynchronous copies requested steps ahead and every global store still in flight.  Here
// the wave's own LDS reads and writes are drained (lgkmcnt) and the waves meet; copies are
// waited for explicitly, by count, where their data is needed.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Inclusive prefix sum of a float over the 64 lanes of a wave with DPP moves (no LDS round trip).
__device__ __forceinline__ float wave_inclusive_scan_f32(float v) {
#define STRD_DPP_FADD(ctrl, row_mask) \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, row_mask, 0xF, true))
    STRD_DPP_FADD(0x111, 0xF);  // row_shr:1
    STRD_DPP_FADD(0x112, 0xF);  // row_shr:2
    STRD_DPP_FADD(0x114, 0xF);  // row_shr:4
    STRD_DPP_FADD(0x118, 0xF);  // row_shr:8
    STRD_DPP_FADD(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
    STRD_DPP_FADD(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef STRD_DPP_FADD
    return v;
}

// Kernels whose LDS tile exceeds the 64 KB default need the limit raised once per (kernel, device);
// a process may drive several devices and call from several threads.
inline bool allow_dynamic_lds(const void *kernel, size_t bytes) {
    constexpr int kMaxDev = 64, kMaxFn = 64;
    static std::mutex mu;
    static const void *fn[kMaxFn];
    static unsigned long long done[kMaxFn];  // bit d: configured on device d
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return false;
    std::lock_guard<std::mutex> lock(mu);
    int slot = -1;
    for (int i = 0; i < kMaxFn; ++i) {
        if (fn[i] == kernel) { slot = i; break; }
        if (!fn[i]) { fn[i] = kernel; slot = i; break; }
    }
    if (slot >= 0 && (done[slot] >> dev & 1ull)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
    if (slot >= 0) done[slot] |= 1ull << dev;
    return true;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? STRD_OK : STRD_EHIP; }

// ---- entry points of the individual kernel files (all enqueue on `s`, return strd_status) ----
int compact_launch(const strd_compact_item *items, int n_items, const int32_t *idx, int N, int M, int K,
                   const int32_t *pos_in, int32_t *pos_out, hipStream_t s);
// packed batches: maxima over the sequences size the grids, the table says what each workgroup owns
int compact_varlen_launch(const strd_compact_item *items, int n_items, const int32_t *idx, const SeqTab &tab, int nseq,
                          int max_rows_out, const int32_t *pos_in, int32_t *pos_out, hipStream_t s);
int select_topk_varlen_max_n();
int select_topk_varlen_launch(const float *scores, int ld, const SeqTab &tab, int nseq, int max_n, int32_t *idx,
                              hipStream_t s);
int score_mamba_general_varlen(const void *B, const void *C, const float *dt, float *s, int ld, const SeqTab &tab, int nseq, int max_n,
                               int H, int G, int n, strd_dtype io, hipStream_t st);
int score_mamba_mfma_varlen(const void *B, const void *C, const float *dt, float *s, int ld, const SeqTab &tab, int nseq, int max_n,
                            int H, int G, int n, void *ws, hipStream_t st);
int score_attn_general_varlen(const void *q, const void *k, float *s, int ld, const SeqTab &tab, int nseq, int max_m,
                              int max_n, int Hq, int Hkv, int d, float scale, strd_dtype io, void *ws, hipStream_t st);
size_t score_attn_mfma_varlen_ws(int nseq, int max_m, int max_n, int Hq, int Hkv);
int score_attn_mfma_varlen(const void *q, const void *k, float *s, int ld, const SeqTab &tab, int nseq, int max_m,
                           int max_n, int Hq, int Hkv, int d, float scale, void *ws, hipStream_t st);
size_t select_topk_ws(int N);
int select_topk_launch(const float *scores, int N, int K, int32_t *idx, void *ws, hipStream_t s);
int select_topk_static_max_n();
int select_topk_static_launch(const float *scores, int N, int K, int32_t *idx, hipStream_t s);

// general SIMT kernels: any shape, fp32 or bf16 I/O, fp32 arithmetic
size_t score_attn_general_ws(int M, int Hq);
int score_attn_general(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, int d,
                       float scale, strd_dtype io, void *ws, hipStream_t st);
int score_mamba_general(const void *B, const void *C, const float *dt, float *s, int M, int N, int H,
                        int G, int n, strd_dtype io, hipStream_t st);
bool ssd_general_supported(int n);
int ssd_general(const void *x, const float *dt, const float *A, const void *B, const void *C,
                const float *D, const float *S_in, void *y, float *S_out, int T, int H, int P, int G,
                int n, strd_dtype io, hipStream_t st);
// bf16 matrix-core paths
bool attn_mfma_supported(int T, int Hq, int Hkv, int d, strd_dtype io);
int attn_mfma(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d, float scale,
              hipStream_t st);
bool score_attn_mfma_supported(int M, int N, int Hq, int Hkv, int d, strd_dtype io);
size_t score_attn_mfma_ws(int M, int N, int Hq, int Hkv);
int score_attn_mfma(const void *q, const void *k, float *s, int M, int N, int Hq, int Hkv, int d, float scale, void *ws,
                    hipStream_t st);
int linear_rocblas(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, strd_dtype io,
                   hipStream_t st);
bool linear_mfma_supported(int T, int Kd, int Nd, strd_dtype io);
int linear_mfma(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, hipStream_t st);
int glue_conv_max_width();
int glue_rmsnorm(const void *x, const void *w, void *out, int T, int d, float eps, strd_dtype io, hipStream_t st);
int glue_gated_rmsnorm(const void *y, const void *z, int ldz, const void *w, void *out, int T, int D, int groups,
                       float eps, strd_dtype io, hipStream_t st);
int glue_conv1d_silu(const void *in, int ld, const void *w, const void *b, void *xo, void *Bo, void *Co, int T, int Cx,
                     int Cb, int W, strd_dtype io, hipStream_t st);
int glue_softplus_dt(const void *raw, int ld, int col0, const float *bias, float *dt, int T, int H, strd_dtype io,
                     hipStream_t st);
int avgpool_launch(const void *src, void *dst, int N, int M, int K, int D, strd_dtype io, const int32_t *pos_in,
                   int32_t *pos_out, hipStream_t st);
int ssd_decode_launch(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
                      float *S, void *y, int H, int P, int G, int n, strd_dtype io, hipStream_t st);
bool attn_decode_supported(int Hq, int Hkv, int d);
size_t attn_decode_workspace(int T, int Hq, int Hkv, int d);
int attn_decode_launch(const void *q, const void *kc, const void *vc, void *o, int T, int Hq, int Hkv, int d,
                       float scale, strd_dtype io, float *ws, hipStream_t st);
bool score_mamba_full_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io);
int score_mamba_full_mfma(const void *B, const void *C, const float *U, const float *V, float *s, int M, int N, int H,
                          int G, int n, void *part_ws, hipStream_t st);
size_t score_mamba_full_ws(int M, int N, int H, int G, int n, strd_dtype io);
int score_mamba_full(const void *B, const void *C, const float *dt_all, const float *A, float *s, int M, int N, int H,
                     int G, int n, strd_dtype io, void *ws, hipStream_t st);
bool score_mamba_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io);
size_t score_mamba_mfma_ws(int N, int G);
int score_mamba_mfma(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, int n,
                     void *ws, hipStream_t st);
bool ssd_seg_supported(int T, int rows, int H, int P, int G, int n, strd_dtype io);
size_t ssd_seg_ws(int T, int H, int P, int G, int n);
bool ssd_seg_preferred(int T, int H, int P, int G);
int ssd_seg(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
            const float *S_in, void *y, float *S_out, const int32_t *idx, int N, int K, int T, int H, int P, int G, int n,
            void *ws, hipStream_t st);
bool ssd_mfma_supported(int T, int rows, int H, int P, int G, int n, strd_dtype io);
int ssd_mfma(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
             const float *S_in, void *y, float *S_out, const int32_t *idx, int N, int K, int T, int H, int P, int G,
             int n, hipStream_t st);

int mfma_rate_probe(float *out, int workgroups, int iters, int mode, hipStream_t st);
bool attn_general_supported(int d);
int attn_general(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d,
                 float scale, strd_dtype io, hipStream_t st);

}  // namespace strd
