// Decode path for 17 to a few hundred rows of X: still bound by streaming W, so W is still read once
// per row block and the MFMA work is hidden behind it.
//
// Same decomposition as the 16-row decode kernel (a workgroup owns 128 columns of W and one K-slice, its
// eight wavefronts take the 32-deep K-blocks round-robin, W blocks are permuted into B operands in
// registers), with one difference: a workgroup carries RG groups of 16 rows (32 or 64 rows of X),
// and every B operand built from W is used for all of them.  More rows than that are further row
// blocks (the grid's z): each re-reads W, which for a few hundred rows is still far cheaper than
// walking K in 64-deep steps with the tiled prefill kernel.
// The reduction across wavefronts (LDS) and across K-slices (workspace, ticket, slice order) is the
// one of the 16-row kernel, run per row group.
// Gated calls with 64 rows per workgroup: the accumulators of four row groups and two weight matrices do
// not fit a wavefront's registers, so the wavefronts split the matrices instead (0-3: W1, 4-7: W2, each
// half taking the K-blocks round-robin); the halves meet in the LDS reduction.  W1 and W2 are still read once.
#include "device_utils.h"
#include "exchange.h"
#include "prism_internal.h"
#include "w_block.h"

#include <type_traits>

namespace prism {

namespace {

constexpr int TN = kDecodeTileN;   // 128
constexpr int KB = kDecodeKBlock;  // 32
constexpr int NW = 8;              // wavefronts per workgroup
constexpr int NT = NW * 64;
constexpr int CPT = 16 * TN / NT;  // 4 columns per thread in the epilogue
constexpr int TPR = TN / CPT;      // 32 threads per output row
constexpr int kRedFloats = NW * 16 * TN;  // one row group's partial tiles of all wavefronts

}  // namespace

// XLDS (calls with one weight matrix): X reaches the wavefront through LDS (see the loop).
template <typename F, bool GATED, int RG, bool XLDS>
__global__ __launch_bounds__(NT) void decode_rows_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ g,
                                                         const uint16_t* __restrict__ W1,
                                                         const uint16_t* __restrict__ W2, uint16_t* __restrict__ Y,
                                                         float* __restrict__ acc_part, float* __restrict__ ss_part,
                                                         unsigned* __restrict__ tickets, int M, int K, int N, float eps,
                                                         int S, int flags) {
    constexpr int G = GATED ? 2 : 1;
    constexpr int RB = 16 * RG;  // rows per workgroup
    constexpr bool HALVES = GATED && RG == 4;  // wavefronts 0-3 take W1, 4-7 take W2
    constexpr bool BOTH = GATED && !HALVES;    // every wavefront takes both matrices
    constexpr int LNW = HALVES ? NW / 2 : NW;  // wavefronts that share one matrix's K-blocks

    extern __shared__ __align__(16) float lds[];  // 16-byte LDS accesses need the alignment said
    float* red = lds;                    // [2][NW][16][TN], reused for every (weight matrix, pair of row groups)
    float* ss_red = lds + 2 * kRedFloats;  // [NW][RB]
    __shared__ int is_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int ntile = blockIdx.x, split = blockIdx.y, rblock = blockIdx.z;
    const int n_tiles = gridDim.x;
    const int n0 = ntile * TN, m0 = rblock * RB;

    const int half = HALVES ? __builtin_amdgcn_readfirstlane(wave / LNW) : 0;
    const int lwave = HALVES ? wave % LNW : wave;

    const int kblocks = (K + KB - 1) / KB;
    const int per = kblocks / S, rem = kblocks % S;
    const int b_beg = split * per + min(split, rem);
    const int b_cnt = per + (split < rem ? 1 : 0);

    const u32 row_bytes = (u32)N * 2u;
    const size_t w_first = (size_t)b_beg * KB * N + n0;
    const size_t w_total = (size_t)K * N;
    const size_t w_left = (w_first < w_total ? w_total - w_first : 0) * 2;
    const u32 w_bytes = (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull);
    const __amdgpu_buffer_rsrc_t rw1 = make_rsrc(((HALVES && half) ? W2 : W1) + w_first, w_bytes);
    const __amdgpu_buffer_rsrc_t rw2 = make_rsrc((GATED ? W2 : W1) + w_first, w_bytes);
    // X from this row block's first row: offsets inside the block stay small whatever M is.
    const size_t x_left = ((size_t)(M - m0) * K) * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + (size_t)m0 * K, (u32)(x_left < 0x7FFFFFFFull ? x_left : 0x7FFFFFFFull));
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(g, (u32)K * 2u);

    const bool col_ok = (n0 + 8 * c) < N;
    const u32 w_lane = col_ok ? ((u32)(8 * q) * row_bytes + (u32)(16 * c)) : kOutOfRange;
    bool row_ok[RG];
    u32 x_row[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        row_ok[r] = (m0 + 16 * r + c) < M;
        x_row[r] = (u32)(16 * r + c) * (u32)K * 2u;
    }

    f32x4 acc1[RG][8], acc2[BOTH ? RG : 1][8];
    float ss[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        ss[r] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc1[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (BOTH) acc2[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }

    // With one row block W is read once and streamed past the caches; several row blocks share it through the L2.
    const bool stream_w = gridDim.z == 1;
    if constexpr (XLDS) {
        static_assert(!GATED, "calls with one weight matrix");
        // A load of X in MFMA operand layout (lane (q, c): row c, eight K values) touches sixteen rows for 64 bytes
        // each, and the compute unit's memory path moves such loads at a third of the rate of loads that take 256
        // contiguous bytes from each of four rows (measured: 17 against 57 bytes per clock).  So a wavefront takes
        // four consecutive K-blocks at a time (128 K values = 256 bytes of a row) and moves their X into an LDS area
        // of its own with buffer loads that have the LDS flag, four rows x 256 bytes per instruction; the operand
        // is then read from LDS.  A load puts lane l's 16 bytes at l * 16 of its 1 KB group; lane l = 16 r + s of
        // group j fetches the eight K values number s ^ (4 j + r) of row 4 j + r, so the sixteen rows of an operand
        // read sit in sixteen different slots (no bank conflicts) and four consecutive lanes still fetch one aligned
        // 64-byte piece.
        typedef __attribute__((address_space(3))) void* lds_ptr;
        u32x4* xs_lane = (u32x4*)lds + (size_t)wave * (RG * 256);
        u32x4* xs_uni = (u32x4*)lds + (size_t)__builtin_amdgcn_readfirstlane(wave) * (RG * 256);
        const int r4 = lane >> 4, slot = lane & 15;
        const int nsb = (b_cnt + 3) / 4;  // super-blocks of four K-blocks in this slice
        const bool gain = (flags & kFlagGain) != 0;
        for (int sb = lwave; sb < nsb; sb += LNW) {
#pragma unroll
            for (int r = 0; r < RG; ++r) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = 16 * r + 4 * j + r4;          // of this workgroup's rows
                    const int oct = slot ^ (4 * j + r4);          // eight K values number oct of the super-block
                    const int ib = 4 * sb + (oct >> 2);
                    const int k = (b_beg + 4 * sb) * KB + 8 * oct;
                    const bool ok = (ib < b_cnt) & (k < K) & (m0 + row < M);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr)(xs_uni + (r * 4 + j) * 64), 16,
                                                             (int)(ok ? (u32)row * (u32)K * 2u + (u32)k * 2u : kOutOfRange), 0, 0, 0);
                }
            }
            // One block at a time (not unrolled: unrolled, the compiler requests all four blocks' W at once and
            // runs out of registers; a second W set in flight under the products was measured and gains nothing).
#pragma unroll 1
            for (int bb = 0; bb < 4; ++bb) {
                const int ib = 4 * sb + bb;
                const bool has = ib < b_cnt;
                const u32 woff = has ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange;
                const int k = (b_beg + ib) * KB + 8 * q;
                WRows w1;
                u32x4 xr[RG];
                const u32x4 gl = load16(rg, (gain & has & (k < K)) ? (u32)k * 2u : kOutOfRange);
                if (stream_w) load_w_block<true>(w1, rw1, woff, row_bytes);
                else load_w_block<false>(w1, rw1, woff, row_bytes);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this super-block's X is in LDS (and W in registers)
#pragma unroll
                for (int r = 0; r < RG; ++r)
                    xr[r] = xs_lane[r * 256 + (c >> 2) * 64 + (c & 3) * 16 + (((4 * bb + q) ^ c) & 15)];
                const u32x4 gr = gain ? gl : ones8<F>();
                u32x4 a[RG];
#pragma unroll
                for (int r = 0; r < RG; ++r) a[r] = scaled_a_operand<F>(xr[r], gr, ss[r]);
                auto step = [&](auto jc) __attribute__((always_inline)) {
                    constexpr int J = decltype(jc)::value;
                    const u32x4 b1 = b_operand<J>(w1);
#pragma unroll
                    for (int r = 0; r < RG; ++r) acc1[r][J] = F::mfma_16x16x32(a[r], b1, acc1[r][J]);
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
        }
        __syncthreads();  // the areas are reused by the reduction below
    } else {
        // U K-blocks per trip: sixteen 16-byte row loads of W in flight per lane where the registers allow it.
        constexpr int U = (!GATED && RG <= 2) ? 2 : 1;
        for (int i = lwave; i < b_cnt; i += U * LNW) {
            WRows w1[U], w2[BOTH ? U : 1];
            u32x4 xr[U][RG], gr[U];
    #pragma unroll
            for (int u = 0; u < U; ++u) {
                const int ib = i + u * LNW;
                const bool has = ib < b_cnt;
                const u32 woff = has ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange;
                const int k = (b_beg + ib) * KB + 8 * q;
                const bool k_ok = has && k < K;
    #pragma unroll
                for (int r = 0; r < RG; ++r)
                    xr[u][r] = load16(rx, (row_ok[r] && k_ok) ? x_row[r] + (u32)k * 2u : kOutOfRange);
                gr[u] = (flags & kFlagGain) ? load16(rg, k_ok ? (u32)k * 2u : kOutOfRange) : ones8<F>();
                if (stream_w) {
                    load_w_block<true>(w1[u], rw1, woff, row_bytes);
                    if (BOTH) load_w_block<true>(w2[u], rw2, woff, row_bytes);
                } else {
                    load_w_block<false>(w1[u], rw1, woff, row_bytes);
                    if (BOTH) load_w_block<false>(w2[u], rw2, woff, row_bytes);
                }
            }
            // Two-matrix calls carry x * g in two parts (scaled_a_operand_split), as in the 16-row kernel.
            auto products = [&](auto split_c) __attribute__((always_inline)) {
                constexpr bool SPLIT = decltype(split_c)::value;
    #pragma unroll
                for (int u = 0; u < U; ++u) {
                    u32x4 a[RG], a_lo[SPLIT ? RG : 1];
    #pragma unroll
                    for (int r = 0; r < RG; ++r) {
                        if constexpr (SPLIT) scaled_a_operand_split<F>(xr[u][r], gr[u], ss[r], a[r], a_lo[r]);
                        else a[r] = scaled_a_operand<F>(xr[u][r], gr[u], ss[r]);
                    }
                    auto step = [&](auto jc) __attribute__((always_inline)) {
                        constexpr int J = decltype(jc)::value;
                        const u32x4 b1 = b_operand<J>(w1[u]);
    #pragma unroll
                        for (int r = 0; r < RG; ++r) {
                            acc1[r][J] = F::mfma_16x16x32(a[r], b1, acc1[r][J]);
                            if constexpr (SPLIT) acc1[r][J] = F::mfma_16x16x32(a_lo[r], b1, acc1[r][J]);
                        }
                        if (BOTH) {
                            const u32x4 b2 = b_operand<J>(w2[BOTH ? u : 0]);
    #pragma unroll
                            for (int r = 0; r < RG; ++r) {
                                acc2[r][J] = F::mfma_16x16x32(a[r], b2, acc2[r][J]);
                                if constexpr (SPLIT) acc2[r][J] = F::mfma_16x16x32(a_lo[r], b2, acc2[r][J]);
                            }
                        }
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
            };
            products(std::integral_constant<bool, GATED>{});
        }
    }

#pragma unroll
    for (int r = 0; r < RG; ++r) {
        ss[r] += __shfl_xor(ss[r], 16, 64);
        ss[r] += __shfl_xor(ss[r], 32, 64);
        if (q == 0) ss_red[wave * RB + 16 * r + c] = ss[r];
    }

    // Epilogue mapping: thread -> (row m of a group, CPT consecutive columns).
    const int m = tid / TPR;
    const int col = (tid % TPR) * CPT;
    const int n = n0 + col;
    bool out_ok[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) out_ok[r] = (m0 + 16 * r + m < M) && (n < N);

    // Across wavefronts through LDS, two row groups of one weight matrix at a time.  Accumulator j, element
    // i of lane (q, c) is row 4q + i of the group, column 8c + j of the tile.
    float v1[RG][CPT], v2[RG][CPT], ssum[RG];
    constexpr int GL = BOTH ? 2 : 1;  // passes over the row groups: one per matrix a wavefront holds
#pragma unroll
    for (int gi = 0; gi < GL; ++gi) {
#pragma unroll
        for (int r0 = 0; r0 < RG; r0 += 2) {
            if (gi + r0 > 0) __syncthreads();
#pragma unroll
            for (int h = 0; h < 2; ++h)
                store_acc_tile(red + h * kRedFloats + wave * 16 * TN, TN, q, c, gi == 0 ? acc1[r0 + h] : acc2[BOTH ? r0 + h : 0]);
            __syncthreads();  // also orders the ss_red stores before their first reader
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = r0 + h;
                float va[CPT], vb[CPT];
#pragma unroll
                for (int e = 0; e < CPT; ++e) { va[e] = 0.f; vb[e] = 0.f; }
                float sq = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float* src = red + h * kRedFloats + (w * 16 + m) * TN + col;
#pragma unroll
                    for (int e = 0; e < CPT; ++e) {
                        if (HALVES && w >= LNW) vb[e] += src[e];
                        else va[e] += src[e];
                    }
                    if (gi == 0 && w < LNW) sq += ss_red[w * RB + 16 * r + m];  // each half has seen all of X
                }
                if (gi == 0) ssum[r] = sq;
#pragma unroll
                for (int e = 0; e < CPT; ++e) {
                    if (gi == 0) v1[r][e] = va[e];
                    else v2[r][e] = va[e];
                    if (HALVES) v2[r][e] = vb[e];
                }
            }
        }
    }
    if (!GATED) {
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int e = 0; e < CPT; ++e) v2[r][e] = 0.f;
    }

    if (S > 1) {
        // Exchange between the K-slices of this (column tile, row block): see the 16-row kernel.
        const size_t tile_id = (size_t)rblock * n_tiles + ntile;
        const __amdgpu_buffer_rsrc_t racc = exchange_rsrc(acc_part, (size_t)S * G * M * N);
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const int row = m0 + 16 * r + m;
            if (out_ok[r]) {
                const size_t idx = (((size_t)split * G) * M + row) * N + n;
                store_partial<CPT>(racc, acc_part, idx, v1[r]);
                if (GATED) store_partial<CPT>(racc, acc_part, idx + (size_t)M * N, v2[r]);
            }
            if (col == 0) store_coherent(ss_part + (tile_id * S + split) * RB + 16 * r + m, ssum[r]);
        }
        wait_stores_acknowledged();
        __syncthreads();
        if (tid == 0) {
            const unsigned prev = __hip_atomic_fetch_add(&tickets[tile_id], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == (unsigned)(S - 1));
        }
        __syncthreads();
        if (!is_last) return;
        if (tid == 0) tickets[tile_id] = 0u;

        // A batch of slices at a time, every row group's loads issued before the first sum; summed in slice order.
        constexpr int BATCH = (RG * G >= 4) ? 4 : 8;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            ssum[r] = 0.f;
#pragma unroll
            for (int e = 0; e < CPT; ++e) { v1[r][e] = 0.f; v2[r][e] = 0.f; }
        }
        for (int s0 = 0; s0 < S; s0 += BATCH) {
            float sq[BATCH][RG];
            float pa[BATCH][RG][CPT], pb[BATCH][GATED ? RG : 1][CPT];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const int s = min(s0 + j, S - 1);
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    sq[j][r] = load_coherent(ss_part + (tile_id * S + s) * RB + 16 * r + m);
                    if (out_ok[r]) {
                        const size_t idx = (((size_t)s * G) * M + (m0 + 16 * r + m)) * N + n;
                        load_partial<CPT>(racc, acc_part, idx, pa[j][r]);
                        if (GATED) load_partial<CPT>(racc, acc_part, idx + (size_t)M * N, pb[j][GATED ? r : 0]);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                if (s0 + j >= S) break;
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    ssum[r] += sq[j][r];
                    if (out_ok[r]) {
#pragma unroll
                        for (int e = 0; e < CPT; ++e) {
                            v1[r][e] += pa[j][r][e];
                            if (GATED) v2[r][e] += pb[j][GATED ? r : 0][e];
                        }
                    }
                }
            }
        }
    }

#pragma unroll
    for (int r = 0; r < RG; ++r) {
        if (!out_ok[r]) continue;
        const float rinv = (flags & kFlagNorm) ? __builtin_amdgcn_rsqf(ssum[r] / (float)K + eps) : 1.0f;
        float y[CPT];
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
            y[e] = v1[r][e] * rinv;
            if (GATED) y[e] = ((flags & kFlagSilu) ? silu_f32(y[e]) : y[e]) * (v2[r][e] * rinv);
        }
        *(u32x2*)(Y + (size_t)(m0 + 16 * r + m) * N + n) = u32x2{F::pack(y[0], y[1]), F::pack(y[2], y[3])};
    }
}

template <typename F, bool GATED, int RG, bool XLDS>
static hipError_t launch_rows(const Call& c, int S, const DecodeWorkspace& ws) {
    const int n_tiles = (c.N + TN - 1) / TN;
    const int row_blocks = (c.M + 16 * RG - 1) / (16 * RG);
    dim3 grid(n_tiles, S, row_blocks), block(NT);
    const size_t lds = (size_t)(2 * kRedFloats + NW * 16 * RG) * sizeof(float);
    auto kern = decode_rows_kernel<F, GATED, RG, XLDS>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c.stream, (const uint16_t*)c.X, (const uint16_t*)c.g,
                       (const uint16_t*)c.W1, (const uint16_t*)(c.gated ? c.W2 : c.W1), (uint16_t*)c.Y, ws.acc_part,
                       ws.ss_part, ws.tickets, c.M, c.K, c.N, c.eps, S, c.flags);
    return hipGetLastError();
}

template <typename F>
static hipError_t launch_rows_fmt(const Call& c, int split_k, int row_groups, bool xlds, const DecodeWorkspace& ws) {
    if (c.gated) {
        if (xlds) return hipErrorInvalidValue;
        if (row_groups == 2) return launch_rows<F, true, 2, false>(c, split_k, ws);
        if (row_groups == 4) return launch_rows<F, true, 4, false>(c, split_k, ws);
    } else {
        if (row_groups == 2) return xlds ? launch_rows<F, false, 2, true>(c, split_k, ws) : launch_rows<F, false, 2, false>(c, split_k, ws);
        if (row_groups == 4) return xlds ? launch_rows<F, false, 4, true>(c, split_k, ws) : launch_rows<F, false, 4, false>(c, split_k, ws);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_decode_rows_16bit(const Call& c, bool f16, int split_k, int row_groups, bool xlds,
                                    const DecodeWorkspace& ws) {
    return f16 ? launch_rows_fmt<F16>(c, split_k, row_groups, xlds, ws)
               : launch_rows_fmt<Bf16>(c, split_k, row_groups, xlds, ws);
}

}  // namespace prism
