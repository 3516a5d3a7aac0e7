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

// Box-Muller: two uniforms -> two independent standard normals (cosine branch first).
__device__ __forceinline__ void box_muller(uint32_t w0, uint32_t w1, float &z0, float &z1)
{
    const float radius = sqrtf(-2.0f * logf(unit_open(w0)));
    float s, c;
    sincospif(2.0f * unit_open(w1), &s, &c);   // angle = 2 pi u, argument reduction is exact
    z0 = radius * c;
    z1 = radius * s;
}

// One thread per Philox block = four consecutive columns of one worker, one 128-bit store.  Threads are
// numbered in storage order (tile, worker, position in tile), so the whole launch writes G front to back.
__global__ void __launch_bounds__(256) synth_grad_kernel(int M, int64_t D, int64_t ld, float sigma, uint64_t seed,
                                                         uint64_t iter, float *__restrict__ G)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // quad index in storage order
    if (t >= (int64_t)M * (ld / 4)) return;
    constexpr int QUADS_PER_TILE = TILE / 4;
    const int64_t tile_row = t / QUADS_PER_TILE;                          // = tile * M + worker
    const int q = (int)(t - tile_row * QUADS_PER_TILE);
    const int64_t tile = tile_row / M;
    const uint32_t i = (uint32_t)(tile_row - tile * M);
    const int64_t j = tile * TILE + (int64_t)q * 4;                       // column of the first element
    const Words4 r = draw_block(seed, STREAM_GRAD, (uint32_t)(j >> 2), i, iter);
    float n0, n1, n2, n3;
    box_muller(r.a, r.b, n0, n1);
    box_muller(r.c, r.d, n2, n3);
    f32x4 z;
    z.x = j + 0 < D ? sigma * n0 : 0.0f;
    z.y = j + 1 < D ? sigma * n1 : 0.0f;
    z.z = j + 2 < D ? sigma * n2 : 0.0f;
    z.w = j + 3 < D ? sigma * n3 : 0.0f;
    store4_stream(G + t * 4, z);
}

void launch_synth_grad(hipStream_t s, int M, int64_t D, int64_t ld, float sigma, uint64_t seed, uint64_t iter,
                       float *G)
{
    const int64_t quads = (int64_t)M * (ld / 4);
    hipLaunchKernelGGL(synth_grad_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, M, D, ld, sigma, seed,
                       iter, G);
}

}  // namespace netmax
