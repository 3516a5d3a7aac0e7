// Consensus distance CD = sum_i ||x_i - mean||^2 (complete-graph form of the penalty in Eq. (1)).
// One pass over X: per column, sums of d and d^2 with d = x_i - x_0 in double (shifting by the first
// row removes the cancellation of the one-pass variance formula), CD_col = sum d^2 - (sum d)^2 / M.
//
// A read-only stream: what matters is how many loads a thread has in flight.  A thread owns CD_VECS groups of four
// columns and walks the workers CD_ROWS at a time: all CD_ROWS x CD_VECS 128-bit loads of a step are requested
// before the first is used.  The sums stay in worker order (the order of the additions does not depend on
// CD_ROWS), so the result is the same double for every choice.  Measured on M = 64 x 11.2 M parameters: 412 us,
// 87 % of the HBM peak (one vector per thread, four rows in flight, cacheable loads: 481 us, 74 %).
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int CD_THREADS = 256;
constexpr int CD_VECS = 2;     // 2 x 256 x 4 columns: a workgroup reads one whole tile, M x 8 KB of contiguous memory
constexpr int CD_ROWS = 8;     // workers whose loads are in flight together
constexpr int CD_COLS = CD_THREADS * 4 * CD_VECS;          // columns per workgroup
static_assert(TILE % CD_COLS == 0, "a workgroup stays inside one tile");
static_assert(CD_COLS % CONSENSUS_COLS == 0, "at most one partial sum per CONSENSUS_COLS columns");

int consensus_partials(int64_t ld) { return (int)((ld + CONSENSUS_COLS - 1) / CONSENSUS_COLS); }
static int consensus_blocks(int64_t ld) { return (int)((ld + CD_COLS - 1) / CD_COLS); }

// every element is read once: non-temporal loads (cacheable ones measured 8 points of the HBM peak slower)
__device__ __forceinline__ f32x4 cd_load(const float *p) { return load4_stream(p); }

__global__ void __launch_bounds__(CD_THREADS)
consensus_partial_kernel(int M, int64_t D, int64_t ld, const float *__restrict__ X, double *__restrict__ partial)
{
    // vector u of this thread covers columns j0 + u * CD_THREADS * 4 .. + 3 (CD_COLS divides TILE: one tile)
    const int64_t j0 = (int64_t)blockIdx.x * CD_COLS + (int64_t)threadIdx.x * 4;
    const float *col = X + tiled_offset(M, 0, j0);                             // worker i is i * TILE further
    double acc = 0.0;
    bool live[CD_VECS];
    f32x4 x0[CD_VECS];
    double s[CD_VECS][4], q[CD_VECS][4];
#pragma unroll
    for (int u = 0; u < CD_VECS; ++u) {
        live[u] = j0 + (int64_t)u * CD_THREADS * 4 < D;
        x0[u] = live[u] ? cd_load(col + u * CD_THREADS * 4) : f32x4{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) s[u][e] = q[u][e] = 0.0;
    }
    for (int i0 = 1; i0 < M; i0 += CD_ROWS) {
        f32x4 r[CD_ROWS][CD_VECS];
#pragma unroll
        for (int k = 0; k < CD_ROWS; ++k)
#pragma unroll
            for (int u = 0; u < CD_VECS; ++u)
                r[k][u] = (live[u] && i0 + k < M) ? cd_load(col + (size_t)(i0 + k) * TILE + u * CD_THREADS * 4) : x0[u];
#pragma unroll
        for (int k = 0; k < CD_ROWS; ++k)
#pragma unroll
            for (int u = 0; u < CD_VECS; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double d = (double)r[k][u][e] - (double)x0[u][e];     // rows past the end read as x_0: d = 0
                    s[u][e] += d;
                    q[u][e] = fma(d, d, q[u][e]);
                }
    }
#pragma unroll
    for (int u = 0; u < CD_VECS; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + (int64_t)u * CD_THREADS * 4 + e < D) acc += q[u][e] - s[u][e] * s[u][e] / (double)M;
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
    const int n = consensus_blocks(ld);
    hipLaunchKernelGGL(consensus_partial_kernel, dim3(n), dim3(CD_THREADS), 0, s, M, D, ld, X, partial);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(CD_THREADS), 0, s, n, partial, out_dev);
}

}  // namespace netmax
