// The fused momentum apply + consensus mix (Eq. (c0), (c1)) restricted to a list of column tiles and with column
// ranges left out: the companion of the weight-gradient kernels that apply the update to their own columns.  It
// covers what those leave (biases, layers they do not handle, the padding, tiles that straddle a boundary).
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

__global__ void __launch_bounds__(256)
mix_subset_kernel(int M, const int32_t *__restrict__ tiles, MixSkip skip, const float *__restrict__ Xcur,
                  const float *__restrict__ G, float *__restrict__ V, float *__restrict__ Xnext,
                  const int32_t *__restrict__ peer, const float *__restrict__ w, float alpha, float mu, float wd)
{
    const unsigned i = blockIdx.x % (unsigned)M;
    const int64_t tile = tiles[blockIdx.x / (unsigned)M];
    int m = peer[i];
    if ((unsigned)m >= (unsigned)M) m = (int)i;
    const float wi = w[(size_t)i * M + m];
    const size_t own = ((size_t)tile * M + i) * TILE, other = ((size_t)tile * M + m) * TILE;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = (u * 256 + (int)threadIdx.x) * 4;
        const int64_t col = tile * TILE + q;
        bool left_out = false;
        for (int r = 0; r < skip.n; ++r) left_out |= (col >= skip.lo[r] && col < skip.hi[r]);
        if (left_out) continue;
        const f32x4 x = load4(Xcur + own + q), xp = load4(Xcur + other + q);
        const f32x4 v = load4_stream(V + own + q), g = load4_stream(G + own + q);
        f32x4 xn, vn;
        momentum_mix4(x, v, g, xp, wi, alpha, mu, wd, xn, vn);
        store4_stream(Xnext + own + q, xn);
        store4_stream(V + own + q, vn);
    }
}

void launch_mix_subset(hipStream_t s, int M, const int32_t *tiles, int n_listed, const MixSkip &skip, const float *Xcur,
                       const float *G, float *V, float *Xnext, const int32_t *peer, const float *w, float alpha, float mu,
                       float wd)
{
    if (n_listed <= 0) return;
    hipLaunchKernelGGL(mix_subset_kernel, dim3((unsigned)n_listed * (unsigned)M), dim3(256), 0, s, M, tiles, skip, Xcur, G, V,
                       Xnext, peer, w, alpha, mu, wd);
}

}  // namespace netmax
