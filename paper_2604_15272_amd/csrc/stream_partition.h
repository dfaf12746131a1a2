// Weighted partition of a decode call's K-blocks over the workgroups of a launch (host and device).
//
// The column tiles of W are laid end to end, tile after tile, each K-block of tile t counting w(t) weight units
// (w_fast, or w_slow for a tile whose columns lie in a slow address slot: tiles repeat their slots with a period
// of 8 or 16 tiles when the row pitch is a multiple of 2 KiB); the T units are cut into G equal consecutive
// ranges, one per workgroup, and a K-block belongs to the workgroup whose range holds its first unit.  A
// workgroup therefore works on a run of K-blocks of one tile, or on the end of one tile and the start of the
// next (paper Table 1: "parallelized matmul (reduction)" with a partition that is uniform in streaming time
// rather than in K), and a tile's partial sums come from consecutive workgroups.  With weights (s, s') and
// G = the sum over the tiles of s or s', every range is a whole share of one tile: a grid of K-slices with s
// slices for most tiles and s' for the slow ones.  All values are exact unsigned 32-bit integers: the host sizes
// the workspace with the same functions the kernel uses.
#pragma once
#include <cstdint>

#include <hip/hip_runtime.h>

namespace prism {

struct StreamPartition {
    uint32_t G;        // workgroups (0: the launch is a plain grid of column tiles x K-slices)
    uint32_t kblocks;  // K-blocks per tile
    uint32_t n_tiles;  // column tiles
    uint32_t slow;     // bit j set: tiles j, j + period, j + 2 period, ... weigh w_slow instead of w_fast
    uint32_t period;   // 8 or 16
    uint32_t w_fast, w_slow;
    uint32_t q, r;     // T = q * G + r
};

constexpr uint32_t kStreamMaxSlices = 32;  // partial sums per tile the kernel can count (half a wavefront)

__host__ __device__ inline uint32_t sp_weight(const StreamPartition& p, uint32_t t) {
    return ((p.slow >> (t & (p.period - 1u))) & 1u) ? p.w_slow : p.w_fast;
}
// Weight units before tile t.
__host__ __device__ inline uint32_t sp_prefix(const StreamPartition& p, uint32_t t) {
    const uint32_t in_period = t & (p.period - 1u), periods = (t - in_period) / p.period;
    const uint32_t slow_before = periods * (uint32_t)__builtin_popcount(p.slow) +
                                 (uint32_t)__builtin_popcount(p.slow & ((1u << in_period) - 1u));
    return (p.w_fast * t + (p.w_slow - p.w_fast) * slow_before) * p.kblocks;
}
// Total weight.
__host__ __device__ inline uint64_t sp_total(const StreamPartition& p) {
    const uint64_t in_period = p.n_tiles & (p.period - 1u), periods = (p.n_tiles - in_period) / p.period;
    const uint64_t slow_tiles = periods * (uint64_t)__builtin_popcount(p.slow) +
                                (uint64_t)__builtin_popcount(p.slow & ((1u << in_period) - 1u));
    return ((uint64_t)p.w_fast * p.n_tiles + (uint64_t)(p.w_slow - p.w_fast) * slow_tiles) * p.kblocks;
}
// First weight unit of workgroup j (j = G: T).  j * r < 2^32 because r < G <= 65535.
__host__ __device__ inline uint32_t sp_boundary(const StreamPartition& p, uint32_t j) {
    return j * p.q + (j * p.r) / p.G;
}
// The tile that holds weight unit v < T.
__host__ __device__ inline uint32_t sp_tile_of(const StreamPartition& p, uint32_t v) {
    const uint32_t u = v / p.kblocks;
    const uint32_t per = p.w_fast * p.period + (p.w_slow - p.w_fast) * (uint32_t)__builtin_popcount(p.slow);
    uint32_t t = (u / per) * p.period, rem = u % per;
    for (uint32_t j = 0; j < p.period; ++j) {
        const uint32_t w = sp_weight(p, t);
        if (rem < w) break;
        rem -= w;
        ++t;
    }
    return t;
}
// K-blocks [r0, r1) of tile t that belong to workgroup j (r0 == r1: none).
__host__ __device__ inline void sp_blocks(const StreamPartition& p, uint32_t j, uint32_t t, uint32_t& r0, uint32_t& r1) {
    const uint32_t lo = sp_boundary(p, j), hi = sp_boundary(p, j + 1), pt = sp_prefix(p, t), w = sp_weight(p, t);
    r0 = lo <= pt ? 0u : (lo - pt + w - 1u) / w;
    r1 = hi <= pt ? 0u : (hi - pt + w - 1u) / w;
    if (r0 > p.kblocks) r0 = p.kblocks;
    if (r1 > p.kblocks) r1 = p.kblocks;
}

}  // namespace prism
