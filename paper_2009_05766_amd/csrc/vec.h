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

// a * b + c per component, one fused multiply-add each.
__device__ __forceinline__ f32x4 fma4(float a, f32x4 b, f32x4 c)
{
    return f32x4{fmaf(a, b[0], c[0]), fmaf(a, b[1], c[1]), fmaf(a, b[2], c[2]), fmaf(a, b[3], c[3])};
}

// Momentum apply and mix of four neighbouring parameters, Eq. (c0) / (c1):
//     v' = mu v + g + wd x,   h = x - alpha v',   x' = h - w (h - x_peer).
// Every kernel that applies the update calls this one function: three fused multiply-adds and one subtraction per
// element in a fixed order, so the kernels agree bit for bit.
__device__ __forceinline__ void momentum_mix4(f32x4 x, f32x4 v, f32x4 g, f32x4 x_peer, float w, float alpha, float mu,
                                              float wd, f32x4 &x_new, f32x4 &v_new)
{
    v_new = fma4(wd, x, fma4(mu, v, g));
    const f32x4 h = fma4(-alpha, v_new, x);
    x_new = fma4(-w, h - x_peer, h);
}

}  // namespace netmax
