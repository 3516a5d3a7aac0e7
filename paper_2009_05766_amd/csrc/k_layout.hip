// Conversion between a plain row-major matrix [M][row_ld] and the worker-interleaved tile layout.
#include "kernels.h"
#include "layout.h"

namespace netmax {

// One thread per element of the tiled matrix, in storage order: tiled[t] = rows[i][j] (0 beyond `cols`).
__global__ void __launch_bounds__(256) pack_kernel(int M, int64_t cols, int64_t ld, const float *__restrict__ rows,
                                                   int64_t row_ld, float *__restrict__ tiled)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)M * ld) return;
    const int64_t tile_row = t >> TILE_SHIFT;
    const int64_t tile = tile_row / M;
    const int i = (int)(tile_row - tile * M);
    const int64_t j = (tile << TILE_SHIFT) + (t & (TILE - 1));
    tiled[t] = j < cols ? rows[(size_t)i * row_ld + j] : 0.0f;
}

// One thread per element of the row-major matrix: rows[i][j] = tiled[...] for j < cols.
__global__ void __launch_bounds__(256) unpack_kernel(int M, int64_t cols, const float *__restrict__ tiled,
                                                     float *__restrict__ rows, int64_t row_ld)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)M * cols) return;
    const int i = (int)(t / cols);
    const int64_t j = t - (int64_t)i * cols;
    rows[(size_t)i * row_ld + j] = tiled[tiled_offset(M, i, j)];
}

// out[k] = the bfloat16 value in[k] widened to float.
__global__ void __launch_bounds__(256) widen_bf16_kernel(int64_t n, const uint16_t *__restrict__ in, float *__restrict__ out)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) out[k] = __uint_as_float((uint32_t)in[k] << 16);
}

void launch_widen_bf16(hipStream_t s, int64_t n, const uint16_t *in, float *out)
{
    hipLaunchKernelGGL(widen_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n, in, out);
}

void launch_pack(hipStream_t s, int M, int64_t cols, int64_t ld, const float *rows, int64_t row_ld, float *tiled)
{
    const int64_t n = (int64_t)M * ld;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, M, cols, ld, rows, row_ld, tiled);
}

void launch_unpack(hipStream_t s, int M, int64_t cols, const float *tiled, float *rows, int64_t row_ld)
{
    const int64_t n = (int64_t)M * cols;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, M, cols, tiled, rows, row_ld);
}

}  // namespace netmax
