// Fused momentum apply + consensus mix (Eq. (c0), (c1)) for all workers: a streaming kernel bound by
// HBM bandwidth.  Per (worker, parameter) it reads x, v, g and the peer's x and writes x' and v'.
//
// One workgroup = one (column tile, worker) pair = 8 KB of each matrix.  In the worker-interleaved tile
// layout the M workgroups of a tile touch one contiguous block per matrix, so walking the tiles in order
// is a linear sweep through HBM.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own
// L2; the id is decoded so that all M workers of a tile run on the same XCD next to each other in time:
// the row a worker pulls from its peer is then fetched from HBM once (by its owner or by the first
// puller) and served from that XCD's L2 afterwards.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int MIX_THREADS = 256;
constexpr int MIX_VECS = TILE / (4 * MIX_THREADS);   // 128-bit accesses per matrix and thread
constexpr int N_XCD = 8;
static_assert(MIX_VECS * 4 * MIX_THREADS == TILE, "a workgroup covers exactly one tile");

__global__ void __launch_bounds__(MIX_THREADS)
mix_kernel(int M, int64_t n_tiles, const float *__restrict__ Xcur, const float *__restrict__ G,
           float *__restrict__ V, float *__restrict__ Xnext, const int32_t *__restrict__ peer,
           const float *__restrict__ w, float alpha, float mu, float wd)
{
    const unsigned bid = blockIdx.x;
    const unsigned xcd = bid % N_XCD, slot = bid / N_XCD;
    const unsigned tile_in_xcd = slot / (unsigned)M;
    const unsigned i = slot - tile_in_xcd * (unsigned)M;
    const int64_t tile = (int64_t)tile_in_xcd * N_XCD + xcd;
    if (tile >= n_tiles) return;

    int m = peer[i];
    if ((unsigned)m >= (unsigned)M) m = (int)i;   // an index outside [0, M) is treated as a self draw
    const float wi = w[(size_t)i * M + m];
    const size_t own = ((size_t)tile * M + i) * TILE, other = ((size_t)tile * M + m) * TILE;
    const float *x = Xcur + own, *xp = Xcur + other, *g = G + own;
    float *v = V + own, *xn = Xnext + own;

    f32x4 rx[MIX_VECS], rp[MIX_VECS], rv[MIX_VECS], rg[MIX_VECS];
#pragma unroll
    for (int u = 0; u < MIX_VECS; ++u) {
        const int j = (u * MIX_THREADS + threadIdx.x) * 4;
        rx[u] = load4(x + j);            // kept cacheable: another worker of this tile may pull this row
        rp[u] = load4(xp + j);
        rv[u] = load4_stream(v + j);
        rg[u] = load4_stream(g + j);
    }
#pragma unroll
    for (int u = 0; u < MIX_VECS; ++u) {
        const int j = (u * MIX_THREADS + threadIdx.x) * 4;
        const f32x4 vn = mu * rv[u] + rg[u] + wd * rx[u];   // v' = mu v + g + wd x
        const f32x4 h = rx[u] - alpha * vn;                 // first-step update
        const f32x4 out = h - wi * (h - rp[u]);             // second-step update towards the peer
        store4_stream(xn + j, out);
        store4_stream(v + j, vn);
    }
}

void launch_mix(hipStream_t s, int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext,
                const int32_t *peer, const float *w, float alpha, float mu, float wd)
{
    const int64_t n_tiles = ld / TILE;
    const int64_t tiles_padded = (n_tiles + N_XCD - 1) / N_XCD * N_XCD;
    hipLaunchKernelGGL(mix_kernel, dim3((unsigned)(tiles_padded * M)), dim3(MIX_THREADS), 0, s, M, n_tiles, Xcur, G, V,
                       Xnext, peer, w, alpha, mu, wd);
}

}  // namespace netmax
