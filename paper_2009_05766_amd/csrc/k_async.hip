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

// The active worker's row: v' = mu v + g + wd x, h = x - alpha v', x' = h - w (h - x_peer), in place.
// One workgroup per column tile (8 KB of the row), 256 threads x 2 x 128 bit.  SYNTH: the gradient of a flat
// model is generated here (and stored to the worker's row of G); otherwise it is read from G.
template <bool SYNTH>
__global__ void __launch_bounds__(256) async_row_kernel(int M, int64_t D, float *__restrict__ X, float *__restrict__ V,
                                                        float *__restrict__ G, const int32_t *__restrict__ active,
                                                        const int32_t *__restrict__ peers, const float *__restrict__ w,
                                                        float alpha, float mu, float wd, float sigma, uint64_t seed, uint64_t k)
{
    const int64_t tile = blockIdx.x;
    int i = *active, m = *peers;
    if ((unsigned)i >= (unsigned)M) return;
    if ((unsigned)m >= (unsigned)M) m = i;
    const float wi = w[(size_t)i * M + m];
    const size_t own = ((size_t)tile * M + i) << TILE_SHIFT, other = ((size_t)tile * M + m) << TILE_SHIFT;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = (u * 256 + (int)threadIdx.x) * 4;
        const f32x4 x = load4(X + own + q), xp = load4(X + other + q), v = load4(V + own + q);
        f32x4 g;
        if (SYNTH) {
            g = synth_grad4(seed, (uint32_t)i, k, tile * TILE + q, D, sigma);
            store4(G + own + q, g);
        } else {
            g = load4(G + own + q);
        }
        f32x4 xn, vn;
        momentum_mix4(x, v, g, xp, wi, alpha, mu, wd, xn, vn);
        store4(X + own + q, xn);
        store4(V + own + q, vn);
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

void launch_async_row(hipStream_t s, bool synth, int M, int64_t D, int64_t ld, float *X, float *V, float *G,
                      const int32_t *active, const int32_t *peers, const float *w, float alpha, float mu, float wd,
                      float sigma, uint64_t seed, uint64_t k)
{
    static_assert(TILE == 2048, "256 threads x 2 x 4 columns cover one tile");
    const dim3 grid((unsigned)(ld / TILE));
    if (synth)
        hipLaunchKernelGGL(async_row_kernel<true>, grid, dim3(256), 0, s, M, D, X, V, G, active, peers, w, alpha, mu, wd, sigma, seed, k);
    else
        hipLaunchKernelGGL(async_row_kernel<false>, grid, dim3(256), 0, s, M, D, X, V, G, active, peers, w, alpha, mu, wd, sigma, seed, k);
}

}  // namespace netmax
