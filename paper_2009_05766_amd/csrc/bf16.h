// bfloat16 helpers: values travel as 16-bit patterns; conversion from float rounds to nearest even.
// The conversions compile to the hardware instruction v_cvt_pk_bf16_f32, which gives the same bits as
// integer round-to-nearest-even (b + 0x7FFF + ((b >> 16) & 1)) >> 16 for every input that is not a NaN
// (all 2^32 patterns compared on the device); a NaN stays a NaN.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace netmax {

typedef float bf_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf_b16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const bf_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf_b16x2));
}
__device__ __forceinline__ uint32_t bf16_bits(float x) { return pack_bf16x2(x, 0.0f) & 0xFFFFu; }
__device__ __forceinline__ float round_bf16(float x) { return __uint_as_float(pack_bf16x2(0.0f, x) & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// a stored bfloat16 activation is positive (ReLU derivative 1)
__device__ __forceinline__ bool bf16_positive(uint16_t h) { return (h & 0x8000u) == 0 && (h & 0x7FFFu) != 0; }

}  // namespace netmax
