// Philox4x32-10 (Salmon et al., SC'11), device code (and the host, which plans the asynchronous schedule's
// batches from the same draws): 4 x u32 counter, 2 x u32 key, ten rounds,
// key bumped by the Weyl constants between rounds.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace netmax {

struct Words4 { uint32_t a, b, c, d; };

__host__ __device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1)
{
    constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    constexpr uint32_t WEYL_0 = 0x9E3779B9u, WEYL_1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        // full 64-bit products: one v_mad_u64_u32 each instead of a high and a low multiply
        const uint64_t prodA = (uint64_t)MUL_A * c0, prodB = (uint64_t)MUL_B * c2;
        const uint32_t t0 = (uint32_t)(prodB >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(prodA >> 32) ^ c3 ^ k1;
        c0 = t0; c1 = (uint32_t)prodB; c2 = t2; c3 = (uint32_t)prodA;
        k0 += WEYL_0; k1 += WEYL_1;
    }
    return Words4{c0, c1, c2, c3};
}

// The iteration number of a draw: a value passed with the launch, or (cell != nullptr) a device cell that a
// replayed HIP graph advances itself, so that the graph's kernel arguments never change.
struct IterRef {
    uint64_t value;
    const uint64_t *cell;
};
__device__ __forceinline__ uint64_t iteration_of(IterRef r) { return r.cell ? *r.cell : r.value; }

// The library's draws: key = (seed_lo, seed_hi ^ stream), counter = (block, worker, iter_lo, iter_hi).
enum : uint32_t { STREAM_PEER = 0u, STREAM_BATCH = 1u, STREAM_GRAD = 2u, STREAM_ACTIVE = 3u };

__host__ __device__ __forceinline__ Words4 draw_block(uint64_t seed, uint32_t stream, uint32_t block, uint32_t worker,
                                             uint64_t iter)
{
    return philox4x32_10(block, worker, (uint32_t)iter, (uint32_t)(iter >> 32), (uint32_t)seed,
                         (uint32_t)(seed >> 32) ^ stream);
}

}  // namespace netmax
