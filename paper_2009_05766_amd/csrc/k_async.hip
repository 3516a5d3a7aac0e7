// The asynchronous schedule of Section II-B / Eq. (c2)-(c4): in global step k one worker i_k is active, drawn
// with the activity probabilities p_i of Eq. (d4); it pulls from m_k ~ P[i_k, :], takes its local step and mixes.
// Only its row of x and v changes, so the update is done in place: x^{k+1} = D^k (x^k - alpha g^k).
#include "kernels.h"
#include "layout.h"
#include "synth.h"

namespace netmax {

// number of thresholds <= u (the first position whose threshold exceeds u), clamped to the last positive entry
__device__ __forceinline__ int search_thresholds(const uint32_t *row, int n, int last, uint32_t u)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row[mid] <= u) lo = mid + 1; else hi = mid;
    }
    return lo < last ? lo : last;
}

// One thread per global step: active[s] = i_k from word 0 of the activity stream at counter (0, 0, k), peers[s] =
// m_k from the peer stream at counter (0, i_k, k), k = first + s.  The draws depend on no state, so all steps of
// a run are drawn by one launch.
__global__ void __launch_bounds__(256) async_draw_kernel(int M, const uint32_t *__restrict__ act_thr, int act_last,
                                                         const uint32_t *__restrict__ thr, const int32_t *__restrict__ last,
                                                         uint64_t seed, uint64_t first, uint64_t n_steps,
                                                         int32_t *__restrict__ active, int32_t *__restrict__ peers)
{
    const uint64_t s = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_steps) return;
    const uint64_t k = first + s;
    const int i = search_thresholds(act_thr, M, act_last, draw_block(seed, STREAM_ACTIVE, 0u, 0u, k).a);
    active[s] = i;
    peers[s] = search_thresholds(thr + (size_t)i * M, M, last[i], draw_block(seed, STREAM_PEER, 0u, (uint32_t)i, k).a);
}

// The active workers' rows of a batch of global steps that do not touch each other's rows (the host plans the
// batches): v' = mu v + g + wd x, h = x - alpha v', x' = h - w (h - x_peer), in place.  One workgroup per column
// tile (8 KB of the row) and step, 256 threads x 2 x 128 bit.  SOURCE 0: the gradient of a flat model is generated
// here with the step's number as iteration and stored to the worker's row of G; 1: it is read from the worker's row
// of G; 2: it is read from slot s of the compact matrix Gc (tile layout over the n_steps slots of the batch) and copied
// to the worker's row of G.
template <int SOURCE>
__global__ void __launch_bounds__(256) async_row_kernel(int M, int64_t D, float *__restrict__ X, float *__restrict__ V,
                                                        float *__restrict__ G, const float *__restrict__ Gc, int n_steps,
                                                        const int32_t *__restrict__ active,
                                                        const int32_t *__restrict__ peers, const float *__restrict__ w,
                                                        float alpha, float mu, float wd, float sigma, uint64_t seed, uint64_t k0)
{
    const int64_t tile = blockIdx.x;
    const int s = blockIdx.y;
    int i = active[s], m = peers[s];
    if ((unsigned)i >= (unsigned)M) return;
    if ((unsigned)m >= (unsigned)M) m = i;
    const float wi = w[(size_t)i * M + m];
    const size_t own = ((size_t)tile * M + i) << TILE_SHIFT, other = ((size_t)tile * M + m) << TILE_SHIFT;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = (u * 256 + (int)threadIdx.x) * 4;
        const f32x4 x = load4(X + own + q), xp = load4(X + other + q), v = load4(V + own + q);
        f32x4 g;
        if (SOURCE == 0) {
            g = synth_grad4(seed, (uint32_t)i, k0 + (uint64_t)s, tile * TILE + q, D, sigma);
            store4(G + own + q, g);
        } else if (SOURCE == 1) {
            g = load4(G + own + q);
        } else {
            g = load4(Gc + (((size_t)tile * n_steps + s) << TILE_SHIFT) + q);
            store4(G + own + q, g);
        }
        f32x4 xn, vn;
        momentum_mix4(x, v, g, xp, wi, alpha, mu, wd, xn, vn);
        store4(X + own + q, xn);
        store4(V + own + q, vn);
    }
}

// Subset runs of the perceptron gradient: the parameter rows of the listed workers copied into a compact matrix
// (tile layout over n slots), their shard descriptors, and their losses copied back.
__global__ void __launch_bounds__(256) gather_rows_kernel(int M, int n, const int32_t *__restrict__ workers,
                                                          const float *__restrict__ X, float *__restrict__ Xc)
{
    const int64_t tile = blockIdx.x;
    const int s = blockIdx.y, i = workers[s];
    if ((unsigned)i >= (unsigned)M) return;
    const size_t src = ((size_t)tile * M + i) << TILE_SHIFT, dst = ((size_t)tile * n + s) << TILE_SHIFT;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = (u * 256 + (int)threadIdx.x) * 4;
        store4(Xc + dst + q, load4(X + src + q));
    }
}

__global__ void __launch_bounds__(256) gather_shards_kernel(int M, int n, const int32_t *__restrict__ workers,
                                                            const int64_t *__restrict__ row0, const int32_t *__restrict__ n_rows,
                                                            int64_t *__restrict__ row0_c, int32_t *__restrict__ n_rows_c)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    int i = workers[s];
    if ((unsigned)i >= (unsigned)M) i = 0;
    row0_c[s] = row0[i];
    n_rows_c[s] = n_rows[i];
}

__global__ void __launch_bounds__(256) scatter_loss_kernel(int M, int n, const int32_t *__restrict__ workers,
                                                           const float *__restrict__ loss_c, float *__restrict__ loss)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    const int i = workers[s];
    if ((unsigned)i < (unsigned)M) loss[i] = loss_c[s];
}

// Batch draws of listed workers: slot s draws for worker workers[s] at iteration first_iter + s (consecutive global
// steps), as sample_batch_kernel does for all workers at one iteration.
__global__ void __launch_bounds__(256) sample_batch_subset_kernel(int n, int B, const int32_t *__restrict__ workers,
                                                                  const int32_t *__restrict__ n_rows_c, uint64_t seed,
                                                                  uint64_t first_iter, int32_t *__restrict__ idx)
{
    const int quads = (B + 3) >> 2;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n * quads) return;
    const int s = t / quads, q = t - s * quads;
    const Words4 r = draw_block(seed, STREAM_BATCH, (uint32_t)q, (uint32_t)workers[s], first_iter + (uint64_t)s);
    const uint32_t rows = (uint32_t)n_rows_c[s];
    const uint32_t wd[4] = {r.a, r.b, r.c, r.d};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int b = 4 * q + e;
        if (b < B) idx[(size_t)s * B + b] = (int32_t)__umulhi(wd[e], rows);
    }
}

// Time bookkeeping (Algorithm 2, UpdateTimeVector) for a run of global steps: one thread per worker walks the steps in
// order and handles those in which it is the active worker, so every worker's entries change in step order.
__global__ void __launch_bounds__(256) async_times_kernel(int M, int64_t n_steps, const int32_t *__restrict__ active,
                                                          const int32_t *__restrict__ peers, const float *__restrict__ t,
                                                          float beta, float *__restrict__ ema, float *__restrict__ clock)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    float c = clock ? clock[i] : 0.0f;
    for (int64_t s = 0; s < n_steps; ++s) {
        if (active[s] != i) continue;
        int m = peers[s];
        if ((unsigned)m >= (unsigned)M) m = i;
        const size_t e = (size_t)i * M + m;
        const float tim = t[e];
        if (m != i) ema[e] = fmaf(beta, ema[e], (1.0f - beta) * tim);
        c += tim;
    }
    if (clock) clock[i] = c;
}

void launch_async_times(hipStream_t s, int M, int64_t n_steps, const int32_t *active, const int32_t *peers, const float *t,
                        float beta, float *ema, float *clock)
{
    hipLaunchKernelGGL(async_times_kernel, dim3((M + 255) / 256), dim3(256), 0, s, M, n_steps, active, peers, t, beta, ema, clock);
}

void launch_async_draw(hipStream_t s, int M, const uint32_t *act_thr, int act_last, const uint32_t *thr, const int32_t *last,
                       uint64_t seed, uint64_t first, uint64_t n_steps, int32_t *active, int32_t *peers)
{
    hipLaunchKernelGGL(async_draw_kernel, dim3((unsigned)((n_steps + 255) / 256)), dim3(256), 0, s, M, act_thr, act_last, thr,
                       last, seed, first, n_steps, active, peers);
}

void launch_async_rows(hipStream_t s, int source, int M, int64_t D, int64_t ld, float *X, float *V, float *G, const float *Gc,
                       int n_steps, const int32_t *active, const int32_t *peers, const float *w, float alpha, float mu, float wd,
                       float sigma, uint64_t seed, uint64_t k0)
{
    static_assert(TILE == 2048, "256 threads x 2 x 4 columns cover one tile");
    const dim3 grid((unsigned)(ld / TILE), (unsigned)n_steps);
    if (source == 0)
        hipLaunchKernelGGL(async_row_kernel<0>, grid, dim3(256), 0, s, M, D, X, V, G, Gc, n_steps, active, peers, w, alpha, mu, wd, sigma, seed, k0);
    else if (source == 1)
        hipLaunchKernelGGL(async_row_kernel<1>, grid, dim3(256), 0, s, M, D, X, V, G, Gc, n_steps, active, peers, w, alpha, mu, wd, sigma, seed, k0);
    else
        hipLaunchKernelGGL(async_row_kernel<2>, grid, dim3(256), 0, s, M, D, X, V, G, Gc, n_steps, active, peers, w, alpha, mu, wd, sigma, seed, k0);
}

void launch_gather_rows(hipStream_t s, int M, int n, int64_t ld, const int32_t *workers, const float *X, float *Xc)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)(ld / TILE), (unsigned)n), dim3(256), 0, s, M, n, workers, X, Xc);
}

void launch_gather_shards(hipStream_t s, int M, int n, const int32_t *workers, const int64_t *row0, const int32_t *n_rows,
                          int64_t *row0_c, int32_t *n_rows_c)
{
    hipLaunchKernelGGL(gather_shards_kernel, dim3((n + 255) / 256), dim3(256), 0, s, M, n, workers, row0, n_rows, row0_c, n_rows_c);
}

void launch_scatter_loss(hipStream_t s, int M, int n, const int32_t *workers, const float *loss_c, float *loss)
{
    hipLaunchKernelGGL(scatter_loss_kernel, dim3((n + 255) / 256), dim3(256), 0, s, M, n, workers, loss_c, loss);
}

void launch_sample_batch_subset(hipStream_t s, int n, int B, const int32_t *workers, const int32_t *n_rows_c, uint64_t seed,
                                uint64_t first_iter, int32_t *idx)
{
    const int total = n * ((B + 3) / 4);
    hipLaunchKernelGGL(sample_batch_subset_kernel, dim3((total + 255) / 256), dim3(256), 0, s, n, B, workers, n_rows_c, seed,
                       first_iter, idx);
}

}  // namespace netmax
