// Decode path: at most 16 rows of X against a large W, bound by streaming W from HBM once.
//
// Work decomposition (paper Table 1: "parallelized matmul (column partition)" across the grid's x,
// "parallelized matmul (reduction)" and the compound parallelized sums across the grid's y, the
// wavefronts of a workgroup and the four lane groups of a wavefront):
//   - a workgroup owns 128 columns of W (and of W2 when gated) and one K-slice;
//   - its wavefronts take the slice's 32-deep K-blocks round-robin;
//   - per K-block a wavefront reads a 32 x 128 piece of W with eight 16-byte loads per lane
//     (lane (q, c), q = lane / 16, c = lane % 16, reads rows 8q..8q+7, columns 8c..8c+7), turns
//     its 8 x 8 sub-block into eight MFMA B operands with byte permutes, and issues eight
//     16x16x32 bf16 MFMAs against the A operand (X * g, rounded to bf16, rows padded to 16);
//   - the raw squares of X are summed per lane in the same loop.
// Afterwards the partial products and partial sums of squares are reduced across wavefronts in
// LDS, and, when the grid splits K, across workgroups through the workspace: every workgroup
// stores its partial, takes a ticket, and the last arrival of a tile sums the partials in slice
// order (so the result does not depend on arrival order), applies 1/rms (and the SiLU gate) and
// stores Y.  The normalised X never exists in memory.
//
// Gated calls come in two tile forms.  Two tiles: a workgroup owns 128 output columns and keeps one accumulator
// tile per weight matrix.  Packed: a workgroup owns 64 output columns, and one 16 x 128 MFMA tile holds their
// products with W1 (lanes c < 8) and with W2 (lanes c >= 8): a row load reads 128 bytes of each matrix, the A
// operand is the same for both, and the gate pairs column j with column 64 + j of the tile.  Twice the tiles,
// so half the K-slices for the same number of workgroups (none at 14336 columns), and half the LDS traffic.
//
// Two ways to deal K out to workgroups: a plain grid (column tiles x S equal K-slices), or the weighted
// partition of stream_partition.h, in which every workgroup of a one-dimensional grid gets the same share of
// streaming time: a run of K-blocks that may end one tile and begin the next (then it makes two passes).
#include "device_utils.h"
#include "exchange.h"
#include "prism_internal.h"
#include "stream_partition.h"
#include "w_block.h"

#include <type_traits>

namespace prism {

namespace {

constexpr int TN = kDecodeTileN;   // 128
constexpr int KB = kDecodeKBlock;  // 32

// The same with the A operand in two parts (scaled_a_operand_split): each B operand is built once and used twice.
template <typename F>
__device__ __forceinline__ void mfma_block_split(f32x4 (&acc)[8], u32x4 a_hi, u32x4 a_lo, const WRows& w) {
    auto step = [&](auto jc) __attribute__((always_inline)) {
        constexpr int J = decltype(jc)::value;
        const u32x4 b = b_operand<J>(w);
        acc[J] = F::mfma_16x16x32(a_hi, b, acc[J]);
        acc[J] = F::mfma_16x16x32(a_lo, b, acc[J]);
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    step(std::integral_constant<int, 4>{});
    step(std::integral_constant<int, 5>{});
    step(std::integral_constant<int, 6>{});
    step(std::integral_constant<int, 7>{});
}

template <typename F>
__device__ __forceinline__ void mfma_block(f32x4 (&acc)[8], u32x4 a, const WRows& w) {
    acc[0] = F::mfma_16x16x32(a, b_operand<0>(w), acc[0]);
    acc[1] = F::mfma_16x16x32(a, b_operand<1>(w), acc[1]);
    acc[2] = F::mfma_16x16x32(a, b_operand<2>(w), acc[2]);
    acc[3] = F::mfma_16x16x32(a, b_operand<3>(w), acc[3]);
    acc[4] = F::mfma_16x16x32(a, b_operand<4>(w), acc[4]);
    acc[5] = F::mfma_16x16x32(a, b_operand<5>(w), acc[5]);
    acc[6] = F::mfma_16x16x32(a, b_operand<6>(w), acc[6]);
    acc[7] = F::mfma_16x16x32(a, b_operand<7>(w), acc[7]);
}

}  // namespace

// LDS: per wavefront a 16 x 128 fp32 tile (two for gated calls with up to eight wavefronts), plus 16 sums of squares.
template <typename F, int NW, bool GATED, bool PACKED = false>
__global__ __launch_bounds__(NW * 64) void decode_kernel(const uint16_t* __restrict__ X,
                                                         const uint16_t* __restrict__ g,
                                                         const uint16_t* __restrict__ W1,
                                                         const uint16_t* __restrict__ W2,
                                                         uint16_t* __restrict__ Y, float* __restrict__ acc_part,
                                                         float* __restrict__ ss_part, unsigned* __restrict__ tickets,
                                                         int M, int K, int N, float eps, int S_grid, int flags,
                                                         StreamPartition sp) {
    constexpr int G = GATED ? 2 : 1;
    constexpr int NT = NW * 64;
    constexpr int CPT = 16 * TN / NT;  // columns per thread in the epilogue (4 for 8 wavefronts)
    constexpr int TPR = TN / CPT;      // threads per output row
    static_assert(CPT >= 2 && CPT <= 8 && (CPT & (CPT - 1)) == 0, "epilogue mapping");
    static_assert(GATED || !PACKED, "the packed tile is a gated tile");
    constexpr int TNO = PACKED ? TN / 2 : TN;  // output columns of a tile

    extern __shared__ __align__(16) float lds[];  // 16-byte LDS accesses need the alignment said
    float* red = lds;                    // [NW][16][TN], used once per weight matrix
    float* ss_red = lds + NW * 16 * TN;  // [NW][16]
    __shared__ int is_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int kblocks = (K + KB - 1) / KB;
    // One pass over a (column tile, run of K-blocks): the tile, the K-blocks [b_beg, b_beg + b_cnt) of it, and this
    // workgroup's place among the S workgroups that share the tile (the order in which the partial sums are
    // added).  Written once, expanded once per pass (a loop over passes would keep both passes' values in
    // registers across its back edge: 256 instead of 168 registers, with spills).
    auto pass = [&](const int ntile, const int split, const int S, const int b_beg, const int b_cnt)
                    __attribute__((always_inline)) {
    const int n0 = ntile * TNO;

    // Buffer descriptors.  W starts at this workgroup's first row and first column; its end is the
    // end of the matrix, so rows past K read as zero.
    const u32 row_bytes = (u32)N * 2u;
    const size_t w_first = (size_t)b_beg * KB * N + n0;
    const size_t w_total = (size_t)K * N;
    const size_t w_left = (w_first < w_total ? w_total - w_first : 0) * 2;
    const u32 w_bytes = (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull);
    const __amdgpu_buffer_rsrc_t rw1 = make_rsrc(W1 + w_first, w_bytes);
    const __amdgpu_buffer_rsrc_t rw2 = make_rsrc((GATED ? W2 : W1) + w_first, w_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X, (u32)((size_t)M * K * 2));
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(g, (u32)K * 2u);

    const int cw = PACKED ? (c & 7) : c;  // this lane's 8-column group inside its matrix's share of the tile
    const bool col_ok = (n0 + 8 * cw) < N;
    const u32 w_lane = col_ok ? ((u32)(8 * q) * row_bytes + (u32)(16 * cw)) : kOutOfRange;
    // Packed: lanes c < 8 read W1, lanes c >= 8 read W2, in one instruction, so through per-lane addresses
    // instead of a descriptor (rows past K and columns past N are predicated off and read as zero).
    const uint16_t* w_ptr = ((PACKED && c >= 8) ? W2 : W1) + ((size_t)b_beg * KB + 8 * q) * N + n0 + 8 * cw;
    const bool row_ok = c < M;

    f32x4 acc1[8], acc2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        acc1[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc2[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float ss = 0.f;

    // U K-blocks per trip, so that sixteen 16-byte row loads of W are in flight per lane.
    constexpr int U = (GATED && !PACKED) ? 1 : 2;
    for (int i = wave; i < b_cnt; i += U * NW) {
        WRows w1[U], w2[U];
        u32x4 xr[U], gr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ib = i + u * NW;
            const bool has = ib < b_cnt;
            const u32 woff = has ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange;
            const int k = (b_beg + ib) * KB + 8 * q;
            const bool k_ok = has && k < K;
            // X and g first: they come from L2 and let the A operand be ready before W lands.
            xr[u] = load16(rx, (row_ok && k_ok) ? (u32)(((size_t)c * K + k) * 2) : kOutOfRange);
            gr[u] = (flags & kFlagGain) ? load16(rg, k_ok ? (u32)k * 2u : kOutOfRange) : ones8<F>();
            if (PACKED) {
                const uint16_t* pw = w_ptr + (size_t)ib * KB * N;
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    w1[u].r[r] = u32x4{0u, 0u, 0u, 0u};
                    if (k_ok && col_ok) w1[u].r[r] = __builtin_nontemporal_load((const u32x4*)(pw + (size_t)r * N));
                }
            } else {
                load_w_block<true>(w1[u], rw1, woff, row_bytes);
                if (GATED) load_w_block<true>(w2[u], rw2, woff, row_bytes);
            }
        }
        // Two-matrix calls carry x * g into the matrix core in two parts: their outputs are products of two sums,
        // and the rounding of x * g to the storage format on either sum, amplified by the other, is what their far
        // tail would otherwise consist of.  The matrix pipe has room (the kernel waits for memory); without a gain
        // the second part is zero.
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (GATED) {
                u32x4 a_hi, a_lo;
                scaled_a_operand_split<F>(xr[u], gr[u], ss, a_hi, a_lo);
                mfma_block_split<F>(acc1, a_hi, a_lo, w1[u]);
                if (!PACKED) mfma_block_split<F>(acc2, a_hi, a_lo, w2[u]);
            } else {
                const u32x4 a = scaled_a_operand<F>(xr[u], gr[u], ss);
                mfma_block<F>(acc1, a, w1[u]);
            }
        }
    }

    // Sum of squares of row c: the four lane groups hold different K values.
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);

    // Epilogue mapping: thread -> (row m, CPT consecutive columns).
    const int m = tid / TPR;
    const int col = (tid % TPR) * CPT;
    const int n = n0 + col;
    // N % 8 == 0 and CPT | 8: all CPT columns valid together.  Packed: the threads of the tile's first 64 columns
    // produce the outputs (each pairs its columns with those 64 further on).
    const bool out_ok = (m < M) && (n < N) && (!PACKED || col < TNO);

    // Reduce across wavefronts through LDS.  Accumulator j, element i of lane (q, c) is row 4q + i, column
    // 8c + j of the tile.  A gated call stores both matrices' tiles at once when LDS holds them (up to eight
    // wavefronts): one barrier instead of three (measured: 44.5 -> 43.3 us on X[8,4096], 2 x W[4096,14336]);
    // otherwise the tile of W2 reuses the space of W1's.
    constexpr bool BOTH_TILES = GATED && (PACKED || NW <= 8);
    float* red2 = PACKED ? red + TNO : red + NW * 16 * TN + NW * 16;  // the tile's second half, or behind ss_red
    float v1[CPT], v2[CPT];
    float ssum = 0.f;
#pragma unroll
    for (int gi = 0; gi < (BOTH_TILES ? 1 : G); ++gi) {
        if (gi == 1) __syncthreads();
        // Rows from M on are padding (zero products): lanes that hold only such rows store nothing, threads that
        // would sum them read nothing (half the LDS traffic with eight rows or fewer).
        if (4 * q < M) {
            store_acc_tile(red + wave * 16 * TN, TN, q, c, gi == 0 ? acc1 : acc2);
            if (BOTH_TILES && !PACKED) store_acc_tile(red2 + wave * 16 * TN, TN, q, c, acc2);
        }
        if (gi == 0 && q == 0) ss_red[wave * 16 + c] = ss;
        __syncthreads();
        float v[CPT], vb[CPT];
#pragma unroll
        for (int e = 0; e < CPT; ++e) { v[e] = 0.f; vb[e] = 0.f; }
        if (m < M && (!PACKED || col < TNO)) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float* src = red + (w * 16 + m) * TN + col;
#pragma unroll
                for (int e = 0; e < CPT; ++e) v[e] += src[e];
                if (BOTH_TILES) {
                    const float* src2 = red2 + (w * 16 + m) * TN + col;
#pragma unroll
                    for (int e = 0; e < CPT; ++e) vb[e] += src2[e];
                }
                if (gi == 0) ssum += ss_red[w * 16 + m];
            }
        }
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
            if (gi == 0) v1[e] = v[e];
            else v2[e] = v[e];
            if (BOTH_TILES) v2[e] = vb[e];
        }
    }
    if (!GATED) {
#pragma unroll
        for (int e = 0; e < CPT; ++e) v2[e] = 0.f;
    }

    if (S > 1) {
        // Publish this slice's partial, then find out whether every other slice has arrived.
        // The partials travel between workgroups that may sit on different XCDs (different L2s).
        // They are written and read with device-coherent accesses (relaxed atomics of agent scope:
        // stores write through, loads do not hit a stale L2 line), so that no whole-cache
        // write-back or invalidate is needed: a workgroup waits until its stores are acknowledged,
        // then takes its ticket; whoever draws the last ticket reads after that.
        const __amdgpu_buffer_rsrc_t racc = exchange_rsrc(acc_part, (size_t)S_grid * G * M * N);
        if (out_ok) {
            const size_t idx = (((size_t)split * G) * M + m) * N + n;
            store_partial<CPT>(racc, acc_part, idx, v1);
            if (GATED) store_partial<CPT>(racc, acc_part, idx + (size_t)M * N, v2);
        }
        if (col == 0) store_coherent(ss_part + ((size_t)ntile * S_grid + split) * 16 + m, ssum);
        wait_stores_acknowledged();
        __syncthreads();
        if (tid == 0) {
            const unsigned prev = __hip_atomic_fetch_add(&tickets[ntile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == (unsigned)(S - 1));
        }
        __syncthreads();
        if (!is_last) return;
        if (tid == 0) tickets[ntile] = 0u;  // ready for the next call on this workspace

        // Eight slices at a time: all their loads are issued before the first sum needs one (a load
        // per trip would cost a round trip to memory per slice); the sums stay in slice order.  Slots
        // past the last slice re-read it and are not added.
        ssum = 0.f;
#pragma unroll
        for (int e = 0; e < CPT; ++e) { v1[e] = 0.f; v2[e] = 0.f; }
        constexpr int BATCH = 8;
        for (int s0 = 0; s0 < S; s0 += BATCH) {
            float sq[BATCH];
            float pa[BATCH][CPT], pb[GATED ? BATCH : 1][CPT];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const int s = min(s0 + j, S - 1);
                sq[j] = load_coherent(ss_part + ((size_t)ntile * S_grid + s) * 16 + m);
                if (out_ok) {
                    const size_t idx = (((size_t)s * G) * M + m) * N + n;
                    load_partial<CPT>(racc, acc_part, idx, pa[j]);
                    if (GATED) load_partial<CPT>(racc, acc_part, idx + (size_t)M * N, pb[GATED ? j : 0]);
                }
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                if (s0 + j >= S) break;
                ssum += sq[j];
                if (out_ok) {
#pragma unroll
                    for (int e = 0; e < CPT; ++e) {
                        v1[e] += pa[j][e];
                        if (GATED) v2[e] += pb[GATED ? j : 0][e];
                    }
                }
            }
        }
    }

    if (!out_ok) return;
    const float rinv = (flags & kFlagNorm) ? __builtin_amdgcn_rsqf(ssum / (float)K + eps) : 1.0f;
    float y[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        y[e] = v1[e] * rinv;
        if (GATED) y[e] = ((flags & kFlagSilu) ? silu_f32(y[e]) : y[e]) * (v2[e] * rinv);
    }
    uint16_t* out = Y + (size_t)m * N + n;
    if (CPT == 1) {
        out[0] = (uint16_t)(F::pack(y[0], 0.f) & 0xFFFFu);
    } else {
        u32 packed[CPT / 2 > 0 ? CPT / 2 : 1];
#pragma unroll
        for (int e = 0; e < CPT / 2; ++e) packed[e] = F::pack(y[2 * e], y[2 * e + 1]);
        if (CPT == 2) *(u32*)out = packed[0];
        if (CPT == 4) *(u32x2*)out = u32x2{packed[0], packed[1]};
        if (CPT == 8) *(u32x4*)out = u32x4{packed[0], packed[1], packed[2], packed[3]};
    }
    };  // pass

    if (sp.G == 0) {
        // Plain grid: column tiles x S_grid equal K-slices.
        const int split = blockIdx.y;
        const int per = kblocks / S_grid, rem = kblocks % S_grid;
        // Workgroups start in the order of their numbers.  With sp.slow set (bit j: column tiles j, j + 8, ... lie in
        // address units that stream slowly; the tile count is a multiple of 8) those tiles get the first numbers: in
        // a launch of several rounds the workgroups that start last then are not the ones that take longest.
        int tile = blockIdx.x;
        if (sp.slow != 0) {
            const uint32_t c_slow = (uint32_t)__builtin_popcount(sp.slow & 0xFFu), n_slow = (gridDim.x >> 3) * c_slow;
            uint32_t pos = blockIdx.x, mask = sp.slow & 0xFFu, c = c_slow;
            if (pos >= n_slow) {
                pos -= n_slow;
                mask ^= 0xFFu;
                c = 8u - c_slow;
            }
            uint32_t nth = pos % c, bit = 0;  // the nth set bit of mask
            for (uint32_t j = 0; j < 8; ++j) {
                const bool set = (mask >> j) & 1u;
                if (set && nth == 0) bit = j;
                nth -= set ? 1u : 0u;
            }
            tile = (int)(8u * (pos / c) + bit);
        }
        pass(tile, split, S_grid, split * per + min(split, rem), per + (split < rem ? 1 : 0));
        return;
    }
    // Weighted partition: this workgroup's range of weight units covers K-blocks of at most two tiles (the host
    // keeps a workgroup's share below a tile's weight).
    const uint32_t v_end = sp_boundary(sp, blockIdx.x + 1);
    const uint32_t t0 = sp_tile_of(sp, sp_boundary(sp, blockIdx.x)), t1 = t0 + 1;
    // A tile's sharers are neighbours in the grid: lane l looks at workgroup blockIdx.x - 32 + l (the host keeps
    // the sharers of a tile at kStreamMaxSlices or fewer).
    const int j = (int)blockIdx.x - 32 + lane;
    const bool j_ok = j >= 0 && j < (int)sp.G;
    uint32_t r0, r1, a0 = 0, a1 = 0;
    sp_blocks(sp, blockIdx.x, t0, r0, r1);
    const bool first = r1 > r0;
    if (first) {
        if (j_ok) sp_blocks(sp, (uint32_t)j, t0, a0, a1);
        const unsigned long long sharers = __ballot(a1 > a0);
        pass((int)t0, __popcll(sharers & 0xFFFFFFFFull), __popcll(sharers), (int)r0, (int)(r1 - r0));
    }
    if (t1 >= sp.n_tiles || sp_prefix(sp, t1) >= v_end) return;
    sp_blocks(sp, blockIdx.x, t1, r0, r1);
    if (r1 <= r0) return;
    a0 = a1 = 0;
    if (j_ok) sp_blocks(sp, (uint32_t)j, t1, a0, a1);
    const unsigned long long sharers = __ballot(a1 > a0);
    if (first) __syncthreads();  // the first pass has finished with LDS
    pass((int)t1, __popcll(sharers & 0xFFFFFFFFull), __popcll(sharers), (int)r0, (int)(r1 - r0));
}

template <typename F, int NW>
static hipError_t launch_decode_nw(const Call& c, int S, const StreamPartition& sp, bool packed,
                                   const DecodeWorkspace& ws) {
    const int tile_cols = packed ? TN / 2 : TN;
    const int n_tiles = (c.N + tile_cols - 1) / tile_cols;
    dim3 grid(n_tiles, S), block(NW * 64);
    if (sp.G != 0) grid = dim3(sp.G);  // S: the most workgroups that share a tile
    const size_t lds = (size_t)(((c.gated && !packed && NW <= 8) ? 2 : 1) * NW * 16 * TN + NW * 16) * sizeof(float);
    auto* X = (const uint16_t*)c.X;
    auto* g = (const uint16_t*)c.g;
    auto* W1 = (const uint16_t*)c.W1;
    auto* W2 = (const uint16_t*)c.W2;
    auto* Y = (uint16_t*)c.Y;
    if (c.gated && packed) {
        if constexpr (NW <= 8) {
            auto kern = decode_kernel<F, NW, true, true>;
            static std::atomic<uint64_t> opted{0};
            if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, grid, block, lds, c.stream, X, g, W1, W2, Y, ws.acc_part, ws.ss_part, ws.tickets,
                               c.M, c.K, c.N, c.eps, S, c.flags, sp);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (c.gated) {
        auto kern = decode_kernel<F, NW, true>;
        static std::atomic<uint64_t> opted{0};
        if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, c.stream, X, g, W1, W2, Y, ws.acc_part, ws.ss_part, ws.tickets,
                           c.M, c.K, c.N, c.eps, S, c.flags, sp);
    } else {
        auto kern = decode_kernel<F, NW, false>;
        static std::atomic<uint64_t> opted{0};
        if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, c.stream, X, g, W1, W1, Y, ws.acc_part, ws.ss_part, ws.tickets,
                           c.M, c.K, c.N, c.eps, S, c.flags, sp);
    }
    return hipGetLastError();
}

template <typename F>
static hipError_t launch_decode_fmt(const Call& c, int split_k, const StreamPartition& sp, int waves, bool packed,
                                    const DecodeWorkspace& ws) {
    switch (waves) {
        case 4: return launch_decode_nw<F, 4>(c, split_k, sp, packed, ws);
        case 8: return launch_decode_nw<F, 8>(c, split_k, sp, packed, ws);
        case 16: return launch_decode_nw<F, 16>(c, split_k, sp, packed, ws);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_decode_16bit(const Call& c, bool f16, int split_k, const StreamPartition& sp, int waves, bool packed,
                               const DecodeWorkspace& ws) {
    return f16 ? launch_decode_fmt<F16>(c, split_k, sp, waves, packed, ws)
               : launch_decode_fmt<Bf16>(c, split_k, sp, waves, packed, ws);
}

}  // namespace prism
