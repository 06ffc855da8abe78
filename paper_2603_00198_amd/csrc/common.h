// Shared device/host helpers for the strd kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

inline int launch_status() { return hipGetLastError() == hipSuccess ? STRD_OK : STRD_EHIP; }

// ---- entry points of the individual kernel files (all enqueue on `s`, return strd_status) ----
int compact_launch(const strd_compact_item *items, int n_items, const int32_t *idx, int N, int M, int K,
                   const int32_t *pos_in, int32_t *pos_out, hipStream_t s);
int select_topk_launch(const float *scores, int N, int K, int32_t *idx, hipStream_t s);

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
bool score_mamba_mfma_supported(int M, int N, int H, int G, int n, strd_dtype io);
int score_mamba_mfma(const void *B, const void *C, const float *dt, float *s, int M, int N, int H, int G, int n,
                     hipStream_t st);
bool ssd_mfma_supported(int T, int H, int P, int G, int n, strd_dtype io);
int ssd_mfma(const void *x, const float *dt, const float *A, const void *B, const void *C, const float *D,
             const float *S_in, void *y, float *S_out, int T, int H, int P, int G, int n, hipStream_t st);

bool attn_general_supported(int d);
int attn_general(const void *q, const void *k, const void *v, void *o, int T, int Hq, int Hkv, int d,
                 float scale, strd_dtype io, hipStream_t st);

}  // namespace strd
