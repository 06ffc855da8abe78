// Measurement aid, not part of the path: the rate at which this chip issues dense bf16 products
// (v_mfma_f32_32x32x16_bf16, or twice as many v_mfma_f32_16x16x32_bf16: the same flops per
// iteration) from registers, with nothing else in the way -- no loads, no LDS, four (eight)
// independent accumulators per wave.  The published peak (2.5 PFLOP/s) assumes the nominal
// clock; under full-rate products the clock follows the power the operands draw, and random bf16
// operands (what real activations look like to the multipliers) draw far more than constants.
// The benchmark reports both rates beside the fraction of the published peak, so that a kernel's
// distance from what the matrix cores can actually sustain on its kind of data is visible.
#include "common.h"

namespace strd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kFrags = 8;  // operand fragments of each kind a wave rotates through

template <bool SMALL>
__global__ __launch_bounds__(kThreads) void mfma_rate_kernel(float *__restrict__ out, int iters, int random_operands) {
    bf16x8 a[kFrags], b[kFrags];
    const unsigned id = blockIdx.x * kThreads + threadIdx.x;
#pragma unroll
    for (int f = 0; f < kFrags; ++f) {
        u32x4 ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // two bf16 per word: random sign and mantissa, exponent of 1.0 (values in +-[1, 2)) -- or 1.0 everywhere
            unsigned h = (id * 2654435761u) ^ ((unsigned)(f * 4 + e) * 40503u + 0x9e3779b9u);
            h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
            unsigned g = h * 0x85ebca6bu; g ^= g >> 16;
            ra[e] = random_operands ? ((h & 0x807F807Fu) | 0x3F803F80u) : 0x3F803F80u;
            rb[e] = random_operands ? ((g & 0x807F807Fu) | 0x3F803F80u) : 0x3F803F80u;
        }
        a[f] = __builtin_bit_cast(bf16x8, ra);
        b[f] = __builtin_bit_cast(bf16x8, rb);
    }
    float t = 0.f;
    if constexpr (SMALL) {
        f32x4 acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int f = 0; f < kFrags; ++f)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[f], b[(f + j + 1) % kFrags], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) t += acc[j][i];
    } else {
        f32x16 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int f = 0; f < kFrags; ++f)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[(f + 2 * j + 1) % kFrags], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) t += acc[j][i];
    }
    out[id] = t;
}

}  // namespace

// flops of one launch: workgroups x 4 waves x iters x 32 products x 32768 (64 products x 16384 in the small form).
// mode: bit 0 = random operands, bit 1 = the 16 x 16 x 32 form of the product
int mfma_rate_probe(float *out, int workgroups, int iters, int mode, hipStream_t st) {
    if (mode & 2)
        mfma_rate_kernel<true><<<workgroups, kThreads, 0, st>>>(out, iters, mode & 1);
    else
        mfma_rate_kernel<false><<<workgroups, kThreads, 0, st>>>(out, iters, mode & 1);
    return launch_status();
}

}  // namespace strd
