// Weighted partition of a decode call's K-blocks over the workgroups of a launch (host and device).
//
// The column tiles of W are laid end to end, tile after tile, each K-block of tile t counting w(t) weight units
// (4, or 5 for a tile whose columns lie in a slow address slot); the T units are cut into G equal consecutive
// ranges, one per workgroup, and a K-block belongs to the workgroup whose range holds its first unit.  A
// workgroup therefore works on a run of K-blocks of one tile, or on the end of one tile and the start of the
// next (paper Table 1: "parallelized matmul (reduction)" with a partition that is uniform in streaming time
// rather than in K), and a tile's partial sums come from consecutive workgroups.  All values are exact unsigned
// 32-bit integers: the host sizes the workspace with the same functions the kernel uses.
#pragma once
#include <cstdint>

#include <hip/hip_runtime.h>

namespace prism {

struct StreamPartition {
    uint32_t G;        // workgroups (0: the launch is a plain grid of column tiles x K-slices)
    uint32_t kblocks;  // K-blocks per tile
    uint32_t n_tiles;  // column tiles
    uint32_t slow;     // bit j set: tiles j, j + 8, j + 16, ... weigh 5 instead of 4
    uint32_t q, r;     // T = q * G + r
};

constexpr uint32_t kStreamMaxSlices = 32;  // partial sums per tile the kernel can count (half a wavefront)

__host__ __device__ inline uint32_t sp_weight(const StreamPartition& p, uint32_t t) {
    return 4u + ((p.slow >> (t & 7u)) & 1u);
}
// Weight units before tile t.
__host__ __device__ inline uint32_t sp_prefix(const StreamPartition& p, uint32_t t) {
    const uint32_t slow_before = (t >> 3) * (uint32_t)__builtin_popcount(p.slow) +
                                 (uint32_t)__builtin_popcount(p.slow & ((1u << (t & 7u)) - 1u));
    return (4u * t + slow_before) * p.kblocks;
}
// First weight unit of workgroup j (j = G: T).  j * r < 2^32 because r < G <= 65535.
__host__ __device__ inline uint32_t sp_boundary(const StreamPartition& p, uint32_t j) {
    return j * p.q + (j * p.r) / p.G;
}
// The tile that holds weight unit v < T.
__host__ __device__ inline uint32_t sp_tile_of(const StreamPartition& p, uint32_t v) {
    const uint32_t u = v / p.kblocks, per8 = 32u + (uint32_t)__builtin_popcount(p.slow);
    uint32_t t = (u / per8) * 8u, rem = u % per8;
    for (int j = 0; j < 8; ++j) {
        const uint32_t w = sp_weight(p, t);
        if (rem < w) break;
        rem -= w;
        ++t;
    }
    return t;
}
// K-blocks [r0, r1) of tile t that belong to workgroup j (r0 == r1: none).
__host__ __device__ inline void sp_blocks(const StreamPartition& p, uint32_t j, uint32_t t, uint32_t& r0, uint32_t& r1) {
    const uint32_t lo = sp_boundary(p, j), hi = sp_boundary(p, j + 1), pt = sp_prefix(p, t);
    const bool five = sp_weight(p, t) == 5u;
    r0 = lo <= pt ? 0u : (five ? (lo - pt + 4u) / 5u : (lo - pt + 3u) >> 2);
    r1 = hi <= pt ? 0u : (five ? (hi - pt + 4u) / 5u : (hi - pt + 3u) >> 2);
    if (r0 > p.kblocks) r0 = p.kblocks;
    if (r1 > p.kblocks) r1 = p.kblocks;
}

}  // namespace prism
