// Synthetic stochastic gradient for flat parameter vectors: g = sigma * N(0,1).  Stands in for a CNN's
// forward/backward pass at the paper's model sizes (Section V-A "Datasets and models").
#include "kernels.h"
#include "layout.h"
#include "synth.h"

namespace netmax {

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
        const f32x4 z = (tile + 1) * TILE <= D ? synth_grad4<true>(seed, i, iter, j, D, sigma)    // the same for the whole workgroup
                                               : synth_grad4<false>(seed, i, iter, j, D, sigma);
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
