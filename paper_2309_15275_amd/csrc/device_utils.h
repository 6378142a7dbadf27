// Small device helpers shared by the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lbp {

// bf16 <-> fp32 on raw bit patterns.  Round-to-nearest-even; inputs here are finite sums of
// finite values, so NaN payload handling is not needed.
__device__ __forceinline__ float bf16_lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// In-register radix-2 Walsh-Hadamard butterfly, natural (Sylvester) order, additions and
// subtractions only.  All indices are compile-time constants after unrolling.
template <int N>
__device__ __forceinline__ void fwht_inplace(float (&v)[N])
{
#pragma unroll
    for (int h = 1; h < N; h <<= 1) {
#pragma unroll
        for (int i = 0; i < N; i += 2 * h) {
#pragma unroll
            for (int j = i; j < i + h; ++j) {
                float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

}  // namespace lbp
