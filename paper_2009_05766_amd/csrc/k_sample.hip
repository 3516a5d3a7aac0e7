// Peer selection (Algorithm 2: "select a neighbor m with probability p_im") and batch draws
// (the sampled dataset D_{i,n} of Eq. (a5)).  Integer work only; results are reproducible bit for bit.
#include "kernels.h"
#include "philox.h"

namespace netmax {

// One thread per worker.  Row i of `thr` holds non-decreasing cumulative thresholds; the peer is the
// number of thresholds <= u (the first m whose threshold exceeds u), clamped to the last positive entry.
__device__ __forceinline__ void draw_peer(int i, int M, const uint32_t *__restrict__ thr, const int32_t *__restrict__ last,
                                          uint64_t seed, uint64_t iter, int32_t *__restrict__ peer)
{
    const uint32_t u = draw_block(seed, STREAM_PEER, 0u, (uint32_t)i, iter).a;
    const uint32_t *row = thr + (size_t)i * M;
    int lo = 0, hi = M;  // upper bound: first position with row[pos] > u
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row[mid] <= u) lo = mid + 1; else hi = mid;
    }
    const int l = last[i];
    peer[i] = lo < l ? lo : l;
}

__global__ void __launch_bounds__(256) sample_peers_kernel(int M, const uint32_t *__restrict__ thr,
                                                           const int32_t *__restrict__ last, uint64_t seed,
                                                           IterRef iter_ref, int32_t *__restrict__ peer)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    draw_peer(i, M, thr, last, seed, iteration_of(iter_ref), peer);
}

// One thread per Philox block of four draws: idx[i][4q..4q+3] = floor(word * n_i / 2^32).
__device__ __forceinline__ void draw_batch_quad(int t, int B, int quads, const int32_t *__restrict__ n_rows, uint64_t seed,
                                                uint64_t iter, int32_t *__restrict__ idx)
{
    const int i = t / quads, q = t - i * quads;
    const Words4 r = draw_block(seed, STREAM_BATCH, (uint32_t)q, (uint32_t)i, iter);
    const uint32_t n = (uint32_t)n_rows[i];
    const uint32_t w[4] = {r.a, r.b, r.c, r.d};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int b = 4 * q + e;
        if (b < B) idx[(size_t)i * B + b] = (int32_t)__umulhi(w[e], n);
    }
}

__global__ void __launch_bounds__(256) sample_batch_kernel(int M, int B, const int32_t *__restrict__ n_rows,
                                                           uint64_t seed, IterRef iter_ref, int32_t *__restrict__ idx)
{
    const int quads = (B + 3) >> 2;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= M * quads) return;
    draw_batch_quad(t, B, quads, n_rows, seed, iteration_of(iter_ref), idx);
}

// Both draws of an iteration in one launch (they are independent): the first peer_blocks workgroups draw the peers,
// the others the batch rows.
__global__ void __launch_bounds__(256) sample_iteration_kernel(int M, const uint32_t *__restrict__ thr,
                                                               const int32_t *__restrict__ last, int32_t *__restrict__ peer,
                                                               int peer_blocks, int B, const int32_t *__restrict__ n_rows,
                                                               int32_t *__restrict__ idx, uint64_t seed, IterRef iter_ref)
{
    const uint64_t iter = iteration_of(iter_ref);
    if ((int)blockIdx.x < peer_blocks) {
        const int i = blockIdx.x * blockDim.x + threadIdx.x;
        if (i < M) draw_peer(i, M, thr, last, seed, iter, peer);
    } else {
        const int quads = (B + 3) >> 2;
        const int t = ((int)blockIdx.x - peer_blocks) * blockDim.x + threadIdx.x;
        if (t < M * quads) draw_batch_quad(t, B, quads, n_rows, seed, iter, idx);
    }
}

void launch_sample_peers(hipStream_t s, int M, const uint32_t *thr, const int32_t *last, uint64_t seed,
                         const IterRef &iter, int32_t *peer)
{
    hipLaunchKernelGGL(sample_peers_kernel, dim3((M + 255) / 256), dim3(256), 0, s, M, thr, last, seed, iter, peer);
}

void launch_sample_batch(hipStream_t s, int M, int B, const int32_t *n_rows, uint64_t seed, const IterRef &iter,
                         int32_t *idx)
{
    const int n = M * ((B + 3) / 4);
    hipLaunchKernelGGL(sample_batch_kernel, dim3((n + 255) / 256), dim3(256), 0, s, M, B, n_rows, seed, iter, idx);
}

void launch_sample_iteration(hipStream_t s, int M, const uint32_t *thr, const int32_t *last, int32_t *peer, int B,
                             const int32_t *n_rows, int32_t *idx, uint64_t seed, const IterRef &iter)
{
    const int peer_blocks = (M + 255) / 256, n = M * ((B + 3) / 4);
    hipLaunchKernelGGL(sample_iteration_kernel, dim3(peer_blocks + (n + 255) / 256), dim3(256), 0, s, M, thr, last, peer,
                       peer_blocks, B, n_rows, idx, seed, iter);
}

// Algorithm 2, UpdateTimeVector, on a simulated network: worker i records the time t[i][m] of its iteration with
// peer m, smooths it into ema[i][m] (exponential moving average) and adds it to its clock.  One thread per worker.
__global__ void __launch_bounds__(256) update_times_kernel(int M, const int32_t *__restrict__ peer,
                                                           const float *__restrict__ t, float beta,
                                                           float *__restrict__ ema, float *__restrict__ clock)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    int m = peer[i];
    if ((unsigned)m >= (unsigned)M) m = i;
    const size_t e = (size_t)i * M + m;
    const float tim = t[e];
    if (m != i) ema[e] = fmaf(beta, ema[e], (1.0f - beta) * tim);
    if (clock) clock[i] += tim;
}

void launch_update_times(hipStream_t s, int M, const int32_t *peer, const float *t, float beta, float *ema, float *clock)
{
    hipLaunchKernelGGL(update_times_kernel, dim3((M + 255) / 256), dim3(256), 0, s, M, peer, t, beta, ema, clock);
}

__global__ void set_iteration_kernel(uint64_t *cell, uint64_t value) { *cell = value; }
__global__ void bump_iteration_kernel(uint64_t *cell) { *cell += 1; }

void launch_set_iteration(hipStream_t s, uint64_t *cell, uint64_t value)
{
    hipLaunchKernelGGL(set_iteration_kernel, dim3(1), dim3(1), 0, s, cell, value);
}
void launch_bump_iteration(hipStream_t s, uint64_t *cell)
{
    hipLaunchKernelGGL(bump_iteration_kernel, dim3(1), dim3(1), 0, s, cell);
}

}  // namespace netmax
