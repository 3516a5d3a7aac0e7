// HBM layout of every per-worker matrix (parameters x, momentum v, gradient g).
//
// Worker-interleaved tiles: the matrix [M workers][ld columns] is cut into column tiles of TILE floats and
// stored as [ld / TILE tiles][M workers][TILE floats].  All M workers' copies of one column tile are then one
// contiguous block of M * 8 KB, so a kernel that walks the tiles in order streams through HBM linearly
// while the rows a worker pulls from its peer sit next to its own (the same block), and a kernel that
// needs one worker's parameters (the gradient GEMMs) finds them as 8 KB pieces at a fixed stride.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace netmax {

constexpr int TILE = 2048;          // floats per tile and worker (8 KB); equals NETMAX_TILE of the C header
constexpr int TILE_SHIFT = 11;
static_assert((1 << TILE_SHIFT) == TILE, "TILE must be a power of two");

// Offset (in floats) of column j of worker i.
__host__ __device__ __forceinline__ size_t tiled_offset(int M, int i, int64_t j)
{
    return (((size_t)(j >> TILE_SHIFT) * (size_t)M + (size_t)i) << TILE_SHIFT) + (size_t)(j & (TILE - 1));
}

}  // namespace netmax
