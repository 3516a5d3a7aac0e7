// The synthetic stochastic gradient of flat parameter vectors, g = sigma * N(0,1): four columns per Philox block.
#pragma once
#include "philox.h"
#include "vec.h"

namespace netmax {

// A 24-bit uniform strictly inside (0,1): ((word >> 9) + 0.5) * 2^-23, exact in single precision.  Two instructions:
// the 23 bits become the mantissa of a number in [1, 2) (the funnel shift supplies the exponent bits), and one
// addition of -(1 - 2^-24) turns it into the value above; both steps are exact.
__device__ __forceinline__ float unit_open(uint32_t word)
{
    const float one_to_two = __builtin_bit_cast(float, __builtin_amdgcn_alignbit(0x7Fu, word, 9u));
    return one_to_two - 0x1.fffffep-1f;
}

// Box-Muller: two uniforms -> two independent standard normals (cosine branch first).  The hardware
// transcendentals are used directly: v_log_f32 is a base-2 logarithm (-2 ln u = -2 ln2 log2 u) and
// v_sin_f32 / v_cos_f32 take their argument in revolutions, so the angle 2 pi u needs no reduction.
// Measured against fp64 over 2.6e8 samples: max abs error 1.1e-6 sigma, the same as logf / sincospif.
__device__ __forceinline__ void box_muller(uint32_t w0, uint32_t w1, float &z0, float &z1)
{
    const float radius = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(unit_open(w0)));
    const float turn = unit_open(w1);
    z0 = radius * __builtin_amdgcn_cosf(turn);
    z1 = radius * __builtin_amdgcn_sinf(turn);
}

// The four gradient values of columns j .. j+3 (j a multiple of 4) of worker i at iteration `iter`; columns
// from D on are padding and get 0.  INSIDE: the caller knows that j + 3 < D (true for whole tiles but the last).
template <bool INSIDE = false>
__device__ __forceinline__ f32x4 synth_grad4(uint64_t seed, uint32_t i, uint64_t iter, int64_t j, int64_t D, float sigma)
{
    const Words4 r = draw_block(seed, STREAM_GRAD, (uint32_t)(j >> 2), i, iter);
    float n0, n1, n2, n3;
    box_muller(r.a, r.b, n0, n1);
    box_muller(r.c, r.d, n2, n3);
    f32x4 z;
    z.x = (INSIDE || j + 0 < D) ? sigma * n0 : 0.0f;
    z.y = (INSIDE || j + 1 < D) ? sigma * n1 : 0.0f;
    z.z = (INSIDE || j + 2 < D) ? sigma * n2 : 0.0f;
    z.w = (INSIDE || j + 3 < D) ? sigma * n3 : 0.0f;
    return z;
}

}  // namespace netmax
