// bfloat16 helpers: values travel as 16-bit patterns; conversion from float rounds to nearest even.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace netmax {

__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    uint32_t b = __float_as_uint(x);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return b >> 16;
}
__device__ __forceinline__ float round_bf16(float x) { return __uint_as_float(bf16_bits(x) << 16); }
__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }
// a stored bfloat16 activation is positive (ReLU derivative 1)
__device__ __forceinline__ bool bf16_positive(uint16_t h) { return (h & 0x8000u) == 0 && (h & 0x7FFFu) != 0; }

}  // namespace netmax
