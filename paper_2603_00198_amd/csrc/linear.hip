// strd_linear: out = x . w (+ residual), the projections of a block -- a plain dense product,
// handed to rocBLAS (bf16 or fp32 storage, fp32 accumulation).  Host code only.
#include <rocblas/rocblas.h>

#include "common.h"

namespace strd {
namespace {

// one rocBLAS handle per device, created on first use and kept for the life of the process
rocblas_handle handle_for_current_device() {
    constexpr int kMaxDev = 64;
    static rocblas_handle handles[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return nullptr;
    if (!handles[dev] && rocblas_create_handle(&handles[dev]) != rocblas_status_success) handles[dev] = nullptr;
    return handles[dev];
}

}  // namespace

int linear_rocblas(const void *x, const void *w, const void *residual, void *out, int T, int Kd, int Nd, strd_dtype io,
                   hipStream_t st) {
    static std::mutex mu;  // a handle carries its stream: one product at a time per process
    std::lock_guard<std::mutex> lock(mu);
    rocblas_handle h = handle_for_current_device();
    if (!h || rocblas_set_stream(h, st) != rocblas_status_success) return STRD_EHIP;
    const rocblas_datatype dt = io == STRD_F32 ? rocblas_datatype_f32_r : rocblas_datatype_bf16_r;
    const float alpha = 1.f, beta = residual ? 1.f : 0.f;
    // row-major out[T, Nd] = x[T, Kd] . w[Kd, Nd]  is column-major  out^T[Nd, T] = w^T[Nd, Kd] . x^T[Kd, T]
    const rocblas_status rc = rocblas_gemm_ex(h, rocblas_operation_none, rocblas_operation_none, Nd, T, Kd, &alpha, w, dt, Nd,
                                              x, dt, Kd, &beta, residual ? residual : out, dt, Nd, out, dt, Nd,
                                              rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    return rc == rocblas_status_success ? STRD_OK : STRD_EHIP;
}

}  // namespace strd
