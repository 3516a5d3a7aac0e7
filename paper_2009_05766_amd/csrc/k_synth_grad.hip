// Synthetic stochastic gradient for flat parameter vectors: g = sigma * N(0,1).  Stands in for a CNN's
// forward/backward pass at the paper's model sizes (Section V-A "Datasets and models").
#include "kernels.h"
#include "layout.h"
#include "synth.h"

namespace netmax {

// A workgroup covers one tile of two neighbouring workers (16 KB, contiguous in the tile layout): every thread
// computes four Philox blocks (two per worker) and only then stores them, so the writes leave in bursts.  Measured
// at 64 workers x 11.2 M columns: 433 us (83 % of the HBM peak, a plain write stream with as many workgroups
// resident reaches 75 %); one block per thread 479 us, eight 517 us.  grid.y strides over the column tiles.
constexpr int SYNTH_WORKERS = 2, SYNTH_THREADS = 256;
static_assert(SYNTH_THREADS * 4 * 2 == TILE, "256 threads x two blocks of 4 columns cover one tile");

__global__ void __launch_bounds__(SYNTH_THREADS)
synth_grad_kernel(int M, int64_t D, int64_t n_tiles, float sigma, uint64_t seed, IterRef iter_ref, float *__restrict__ G)
{
    const uint64_t iter = iteration_of(iter_ref);
    const uint32_t i0 = blockIdx.x * SYNTH_WORKERS;
    const int q = (int)threadIdx.x;                                          // first of the thread's two quads of a tile
    for (int64_t tile = blockIdx.y; tile < n_tiles; tile += gridDim.y) {
        f32x4 z[SYNTH_WORKERS][2];
        const bool inside = (tile + 1) * TILE <= D;                          // no padding in this tile
#pragma unroll
        for (int wk = 0; wk < SYNTH_WORKERS; ++wk)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int64_t j = tile * TILE + (int64_t)(q + SYNTH_THREADS * h) * 4;   // column of the first element
                z[wk][h] = inside ? synth_grad4<true>(seed, i0 + wk, iter, j, D, sigma)
                                  : synth_grad4<false>(seed, i0 + wk, iter, j, D, sigma);
            }
#pragma unroll
        for (int wk = 0; wk < SYNTH_WORKERS; ++wk)
            if (i0 + wk < (uint32_t)M)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    store4_stream(G + (((size_t)tile * M + i0 + wk) << TILE_SHIFT) + (q + SYNTH_THREADS * h) * 4, z[wk][h]);
    }
}

void launch_synth_grad(hipStream_t s, int M, int64_t D, int64_t ld, float sigma, uint64_t seed, const IterRef &iter,
                       float *G)
{
    const int64_t n_tiles = ld / TILE;
    const unsigned gy = (unsigned)(n_tiles < 65535 ? n_tiles : 65535);
    hipLaunchKernelGGL(synth_grad_kernel, dim3((unsigned)((M + SYNTH_WORKERS - 1) / SYNTH_WORKERS), gy), dim3(SYNTH_THREADS), 0, s,
                       M, D, n_tiles, sigma, seed, iter, G);
}

}  // namespace netmax
