// Fused momentum apply + consensus mix (Eq. (c0), (c1)) for all workers: a streaming kernel bound by
// HBM bandwidth.  Per (worker, parameter) it reads x, v, g and the peer's x and writes x' and v'.
//
// Work decomposition: one workgroup = one worker row x one column chunk of CHUNK floats.  Workgroups
// are numbered so that (a) all M rows of a column chunk are dispatched next to each other, and
// (b) they land on the same XCD (workgroup ids are dealt round-robin to the 8 XCDs), so the row a
// worker pulls from its peer is fetched from HBM once and served from that XCD's L2 the second time.
#include "kernels.h"
#include "vec.h"

namespace netmax {

constexpr int MIX_THREADS = 256;
constexpr int MIX_UNROLL = 4;                               // 128-bit accesses in flight per stream and thread
constexpr int MIX_CHUNK = MIX_THREADS * 4 * MIX_UNROLL;     // floats per workgroup
constexpr int N_XCD = 8;

__global__ void __launch_bounds__(MIX_THREADS)
mix_kernel(int M, int64_t ld, const float *__restrict__ Xcur, const float *__restrict__ G, float *__restrict__ V,
           float *__restrict__ Xnext, const int32_t *__restrict__ peer, const float *__restrict__ w, float alpha,
           float mu, float wd)
{
    const unsigned bid = blockIdx.x;
    const unsigned xcd = bid % N_XCD, slot = bid / N_XCD;
    const unsigned chunk_in_xcd = slot / (unsigned)M;
    const unsigned i = slot - chunk_in_xcd * (unsigned)M;
    const int64_t base = ((int64_t)chunk_in_xcd * N_XCD + xcd) * MIX_CHUNK;
    if (base >= ld) return;

    int m = peer[i];
    if ((unsigned)m >= (unsigned)M) m = (int)i;   // an index outside [0, M) is treated as a self draw
    const float wi = w[(size_t)i * M + m];
    const float *x = Xcur + (size_t)i * ld, *xp = Xcur + (size_t)m * ld, *g = G + (size_t)i * ld;
    float *v = V + (size_t)i * ld, *xn = Xnext + (size_t)i * ld;

    f32x4 rx[MIX_UNROLL], rp[MIX_UNROLL], rv[MIX_UNROLL], rg[MIX_UNROLL];
#pragma unroll
    for (int u = 0; u < MIX_UNROLL; ++u) {
        const int64_t j = base + ((int64_t)u * MIX_THREADS + threadIdx.x) * 4;
        if (j < ld) {
            rx[u] = load4(x + j);
            rp[u] = load4(xp + j);
            rv[u] = load4_stream(v + j);
            rg[u] = load4_stream(g + j);
        }
    }
#pragma unroll
    for (int u = 0; u < MIX_UNROLL; ++u) {
        const int64_t j = base + ((int64_t)u * MIX_THREADS + threadIdx.x) * 4;
        if (j < ld) {
            const f32x4 vn = mu * rv[u] + rg[u] + wd * rx[u];   // v' = mu v + g + wd x
            const f32x4 h = rx[u] - alpha * vn;                 // first-step update
            const f32x4 out = h - wi * (h - rp[u]);             // second-step update towards the peer
            store4_stream(xn + j, out);
            store4_stream(v + j, vn);
        }
    }
}

void launch_mix(hipStream_t s, int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext,
                const int32_t *peer, const float *w, float alpha, float mu, float wd)
{
    const int64_t chunks = (ld + MIX_CHUNK - 1) / MIX_CHUNK;
    const int64_t chunks_padded = (chunks + N_XCD - 1) / N_XCD * N_XCD;
    hipLaunchKernelGGL(mix_kernel, dim3((unsigned)(chunks_padded * M)), dim3(MIX_THREADS), 0, s, M, ld, Xcur, G, V,
                       Xnext, peer, w, alpha, mu, wd);
}

}  // namespace netmax
