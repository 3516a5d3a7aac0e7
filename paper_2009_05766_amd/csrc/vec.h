// 128-bit vector type for global loads/stores and cache-policy helpers.
#pragma once
#include <hip/hip_runtime.h>

namespace netmax {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 load4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ f32x4 load4_stream(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
}
__device__ __forceinline__ void store4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
__device__ __forceinline__ void store4_stream(float *p, f32x4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(p));
}

}  // namespace netmax
