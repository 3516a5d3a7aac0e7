// Synthetic stochastic gradient for flat parameter vectors: g = sigma * N(0,1).  Stands in for a CNN's
// forward/backward pass at the paper's model sizes (Section V-A "Datasets and models").
#include "kernels.h"
#include "layout.h"
#include "philox.h"
#include "vec.h"

namespace netmax {

// A 24-bit uniform strictly inside (0,1): ((word >> 9) + 0.5) * 2^-23, exact in single precision.
__device__ __forceinline__ float unit_open(uint32_t word)
{
    return (float)(word >> 9) * 0x1p-23f + 0x1p-24f;
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

// One thread per Philox block = four consecutive columns of one worker, one 128-bit store.
// grid.x = 2 M: workgroup (worker, half tile); grid.y strides over the column tiles, so consecutive
// workgroups write consecutive 4 KB pieces of G and no thread needs a division.
__global__ void __launch_bounds__(256) synth_grad_kernel(int M, int64_t D, int64_t n_tiles, float sigma, uint64_t seed,
                                                         IterRef iter_ref, float *__restrict__ G)
{
    const uint64_t iter = iteration_of(iter_ref);
    const uint32_t i = blockIdx.x >> 1;
    const int q = (int)(blockIdx.x & 1) * 256 + (int)threadIdx.x;            // quad inside the tile
    for (int64_t tile = blockIdx.y; tile < n_tiles; tile += gridDim.y) {
        const int64_t j = tile * TILE + (int64_t)q * 4;                      // column of the first element
        const Words4 r = draw_block(seed, STREAM_GRAD, (uint32_t)(j >> 2), i, iter);
        float n0, n1, n2, n3;
        box_muller(r.a, r.b, n0, n1);
        box_muller(r.c, r.d, n2, n3);
        f32x4 z;
        z.x = j + 0 < D ? sigma * n0 : 0.0f;
        z.y = j + 1 < D ? sigma * n1 : 0.0f;
        z.z = j + 2 < D ? sigma * n2 : 0.0f;
        z.w = j + 3 < D ? sigma * n3 : 0.0f;
        store4_stream(G + (((size_t)tile * M + i) << TILE_SHIFT) + q * 4, z);
    }
}

void launch_synth_grad(hipStream_t s, int M, int64_t D, int64_t ld, float sigma, uint64_t seed, const IterRef &iter,
                       float *G)
{
    static_assert(TILE == 2048, "two workgroups of 256 threads x 4 columns cover one tile");
    const int64_t n_tiles = ld / TILE;
    const unsigned gy = (unsigned)(n_tiles < 65535 ? n_tiles : 65535);
    hipLaunchKernelGGL(synth_grad_kernel, dim3(2 * M, gy), dim3(256), 0, s, M, D, n_tiles, sigma, seed, iter, G);
}

}  // namespace netmax
