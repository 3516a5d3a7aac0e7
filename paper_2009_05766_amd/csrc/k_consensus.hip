// Consensus distance CD = sum_i ||x_i - mean||^2 (complete-graph form of the penalty in Eq. (1)).
// One pass over X: per column, sums of d and d^2 with d = x_i - x_0 in double (shifting by the first
// row removes the cancellation of the one-pass variance formula), CD_col = sum d^2 - (sum d)^2 / M.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int CD_THREADS = 256;
constexpr int CD_COLS = CD_THREADS * 4;
static_assert(CD_COLS == CONSENSUS_COLS, "one partial sum per CONSENSUS_COLS columns");
static_assert(TILE % CD_COLS == 0, "a workgroup stays inside one tile");

int consensus_partials(int64_t ld) { return (int)((ld + CD_COLS - 1) / CD_COLS); }

__global__ void __launch_bounds__(CD_THREADS)
consensus_partial_kernel(int M, int64_t D, int64_t ld, const float *__restrict__ X, double *__restrict__ partial)
{
    const int64_t j = ((int64_t)blockIdx.x * CD_THREADS + threadIdx.x) * 4;   // CD_COLS divides TILE
    double acc = 0.0;
    if (j < D) {
        const float *col = X + tiled_offset(M, 0, j);                          // worker i is i * TILE further
        const f32x4 x0 = load4(col);
        double s[4] = {0, 0, 0, 0}, q[4] = {0, 0, 0, 0};
#pragma unroll 4
        for (int i = 1; i < M; ++i) {
            const f32x4 xi = load4(col + (size_t)i * TILE);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = (double)xi[e] - (double)x0[e];
                s[e] += d;
                q[e] = fma(d, d, q[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j + e < D) acc += q[e] - s[e] * s[e] / (double)M;
    }
    // workgroup reduction in a fixed order
    __shared__ double red[CD_THREADS];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int stride = CD_THREADS / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) red[threadIdx.x] += red[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(CD_THREADS) consensus_final_kernel(int n, const double *__restrict__ partial,
                                                                     double *__restrict__ out)
{
    __shared__ double red[CD_THREADS];
    double acc = 0.0;
    for (int k = threadIdx.x; k < n; k += CD_THREADS) acc += partial[k];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int stride = CD_THREADS / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) red[threadIdx.x] += red[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = red[0];
}

void launch_consensus(hipStream_t s, int M, int64_t D, int64_t ld, const float *X, double *partial, double *out_dev)
{
    const int n = consensus_partials(ld);
    hipLaunchKernelGGL(consensus_partial_kernel, dim3(n), dim3(CD_THREADS), 0, s, M, D, ld, X, partial);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(CD_THREADS), 0, s, n, partial, out_dev);
}

}  // namespace netmax
