// Fused momentum apply + consensus mix (Eq. (c0), (c1)) for all workers: a streaming kernel bound by
// HBM bandwidth.  Per (worker, parameter) it reads x, v, g and the peer's x and writes x' and v'.
//
// A slot = one (column tile, worker) pair = 8 KB of each matrix.  In the worker-interleaved tile layout the M slots
// of a tile are one contiguous block per matrix, so walking the slots in order is a linear sweep through HBM.
// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2; the id is decoded so that all M workers
// of a tile run on the same XCD next to each other in time: the row a worker pulls from its peer is then fetched
// from HBM once (by its owner or by the first puller) and served from that XCD's L2 afterwards.
//
// How much a compute unit has in flight decides the rate.  Large problems run one workgroup per compute unit that
// covers four neighbouring slots (two groups of 256 threads, two slots each), requests all its loads, waits for
// them together and only then stores: the memory controllers see bursts of reads and bursts of writes of a few
// streams instead of many interleaved ones.  Measured on M = 64 x 11.2 M parameters: 78 to 79 % of the HBM peak,
// against 73 % for one slot per workgroup with as many workgroups resident as fit (77 % with two resident).
// Small problems (a few slots per compute unit) and small worker counts keep the one-slot form.
#include "kernels.h"
#include "layout.h"
#include "vec.h"

namespace netmax {

constexpr int MIX_LANES = 256;                     // threads that cover one slot
constexpr int MIX_VECS = TILE / (4 * MIX_LANES);   // 128-bit accesses per matrix, slot and thread
constexpr int N_XCD = 8;
static_assert(MIX_VECS * 4 * MIX_LANES == TILE, "256 threads cover exactly one tile");
// the large form asks for a whole compute unit's LDS (never touched): one resident workgroup per compute unit
constexpr unsigned MIX_LDS_BYTES = 160 * 1024 - 512;
constexpr int64_t MIX_SMALL_SLOTS = 16384;         // below this many slots: the one-slot form
constexpr int MIX_SMALL_M = 32;                    // and below this many workers (measured: 5 % slower there at M = 8, 16)

template <int SLOTS, int GROUPS, bool GATHERED>
__global__ void __launch_bounds__(MIX_LANES * GROUPS)
mix_kernel(int M, int64_t n_tiles, const float *__restrict__ Xcur, const float *__restrict__ G,
           float *__restrict__ V, float *__restrict__ Xnext, const int32_t *__restrict__ peer,
           const float *__restrict__ w, float alpha, float mu, float wd)
{
    const unsigned bid = blockIdx.x;
    const unsigned xcd = bid % N_XCD, lane = threadIdx.x % MIX_LANES, group = threadIdx.x / MIX_LANES;
    // slots of this XCD in sweep order: slot = tile_in_xcd * M + worker; this group takes SLOTS neighbouring ones
    const unsigned slot0 = ((bid / N_XCD) * GROUPS + group) * SLOTS;

    f32x4 rx[SLOTS][MIX_VECS], rp[SLOTS][MIX_VECS], rv[SLOTS][MIX_VECS], rg[SLOTS][MIX_VECS];
    size_t own[SLOTS], other[SLOTS];
    float wi[SLOTS];
    bool live[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const unsigned slot = slot0 + s, tile_in_xcd = slot / (unsigned)M, i = slot - tile_in_xcd * (unsigned)M;
        const int64_t tile = (int64_t)tile_in_xcd * N_XCD + xcd;
        live[s] = tile < n_tiles;
        int m = live[s] ? peer[i] : 0;
        if ((unsigned)m >= (unsigned)M) m = (int)i;       // an index outside [0, M) is treated as a self draw
        wi[s] = live[s] ? w[(size_t)i * M + m] : 0.0f;
        own[s] = live[s] ? ((size_t)tile * M + i) * TILE : 0;
        other[s] = live[s] ? ((size_t)tile * M + m) * TILE : 0;
    }
    // Requests go out matrix by matrix over all slots of the group (x, v, g, then the peers' rows), not slot by
    // slot: measured 1.5 points of the HBM peak better with several slots per group.
    const int j0 = (int)lane * 4;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u)
                rx[s][u] = load4(Xcur + own[s] + u * MIX_LANES * 4 + j0);    // kept cacheable: another worker of this tile may pull this row
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u) rv[s][u] = load4_stream(V + own[s] + u * MIX_LANES * 4 + j0);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u) rg[s][u] = load4_stream(G + own[s] + u * MIX_LANES * 4 + j0);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u) rp[s][u] = load4(Xcur + other[s] + u * MIX_LANES * 4 + j0);
    if (GATHERED) {
        // every load of the workgroup has arrived before its first store leaves
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0), the other counters untouched
        __syncthreads();
    }
    f32x4 xo[SLOTS][MIX_VECS], vo[SLOTS][MIX_VECS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
        for (int u = 0; u < MIX_VECS; ++u)
            momentum_mix4(rx[s][u], rv[s][u], rg[s][u], rp[s][u], wi[s], alpha, mu, wd, xo[s][u], vo[s][u]);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u) store4_stream(Xnext + own[s] + u * MIX_LANES * 4 + j0, xo[s][u]);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        if (live[s])
#pragma unroll
            for (int u = 0; u < MIX_VECS; ++u) store4_stream(V + own[s] + u * MIX_LANES * 4 + j0, vo[s][u]);
}

void launch_mix(hipStream_t s, int M, int64_t ld, const float *Xcur, const float *G, float *V, float *Xnext,
                const int32_t *peer, const float *w, float alpha, float mu, float wd)
{
    const int64_t n_tiles = ld / TILE;
    const int64_t slots_per_xcd = (n_tiles + N_XCD - 1) / N_XCD * M;
    if (n_tiles * M < MIX_SMALL_SLOTS || M < MIX_SMALL_M) {
        hipLaunchKernelGGL((mix_kernel<1, 1, false>), dim3((unsigned)(slots_per_xcd * N_XCD)), dim3(MIX_LANES), 0, s, M,
                           n_tiles, Xcur, G, V, Xnext, peer, w, alpha, mu, wd);
    } else {
        const int64_t groups_of_four = (slots_per_xcd + 3) / 4;
        hipLaunchKernelGGL((mix_kernel<2, 2, true>), dim3((unsigned)(groups_of_four * N_XCD)), dim3(2 * MIX_LANES),
                           MIX_LDS_BYTES, s, M, n_tiles, Xcur, G, V, Xnext, peer, w, alpha, mu, wd);
    }
}

hipError_t prepare_mix()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(mix_kernel<2, 2, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)MIX_LDS_BYTES);
}

}  // namespace netmax
