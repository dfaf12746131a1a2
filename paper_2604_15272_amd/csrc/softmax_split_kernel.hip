// Softmax followed by a matrix product with K split across workgroups (paper Figure 1; Table 1,
// "parallelized matmul (reduction)" and the compound parallelized sums).
//
// The kernel that gives a workgroup 16 rows over the whole of K makes every workgroup read all of its
// 128 columns of W: at the paper's shape (X[4096,4096], W[4096,128]) that is 1 MiB of W per 128 KiB of X
// through one compute unit's vector-memory path (64 bytes per clock), which then sets the time, not HBM.
// Here a workgroup owns 32 rows, 128 columns and one K-slice: every B operand built from W serves two
// groups of 16 rows, and with S slices a workgroup reads 1/S of W, while row blocks x slices still fill the
// chip.  A wavefront walks its K-blocks once, with a running row maximum (accumulators rescaled when it
// moves), as the 16-row kernel does.  What a workgroup hands over is (maximum, sum of exponentials,
// partial product) relative to the slice's own maximum, and the last arrival of a tile (atomic ticket)
// rescales every slice to the common maximum, adds them in slice order and divides: the same algebra as the
// division after the loop in Figure 1(b), applied once more across slices.
#include <type_traits>

#include "device_utils.h"
#include "exchange.h"
#include "prism_internal.h"
#include "w_block.h"

namespace prism {

namespace {

constexpr int TN = kSoftmaxTileN;  // 128
constexpr int KB = 32;
constexpr int NW = 8;
constexpr int NT = NW * 64;
constexpr int RG = 2;             // 16-row groups per workgroup
constexpr int RB = 16 * RG;       // rows per workgroup
constexpr int CPT = 16 * TN / NT;  // 4 columns per thread in the epilogue
constexpr int TPR = TN / CPT;      // 32 threads per output row
constexpr int kRedFloats = NW * 16 * TN;
constexpr float kLog2e = 1.4426950408889634f;

}  // namespace

template <typename F>
__global__ __launch_bounds__(NT) void softmax_split_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ W,
                                                           uint16_t* __restrict__ Y, float* __restrict__ acc_part,
                                                           float* __restrict__ ml_part, unsigned* __restrict__ tickets,
                                                           int M, int K, int N, int S) {
    extern __shared__ __align__(16) float lds[];  // 16-byte LDS accesses need the alignment said
    float* red = lds;                       // [RG][NW][16][TN]
    float* wave_max = lds + RG * kRedFloats;  // [NW][RB]
    float* wave_sum = wave_max + NW * RB;     // [NW][RB]
    __shared__ int is_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int ntile = blockIdx.x, split = blockIdx.y, rblock = blockIdx.z;
    const int n_tiles = gridDim.x;
    const int n0 = ntile * TN, m0 = rblock * RB;

    // This workgroup's K-blocks: [b_beg, b_beg + b_cnt).
    const int kblocks = (K + KB - 1) / KB;
    const int per = kblocks / S, rem = kblocks % S;
    const int b_beg = split * per + min(split, rem);
    const int b_cnt = per + (split < rem ? 1 : 0);

    const size_t x_left = ((size_t)(M - m0) * K) * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + (size_t)m0 * K, (u32)(x_left < 0x7FFFFFFFull ? x_left : 0x7FFFFFFFull));
    const size_t w_first = (size_t)b_beg * KB * N + n0;
    const size_t w_total = (size_t)K * N;
    const size_t w_left = (w_first < w_total ? w_total - w_first : 0) * 2;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(W + w_first, (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull));
    const u32 row_bytes = (u32)N * 2u;
    const bool col_ok = (n0 + 8 * c) < N;
    const u32 w_lane = col_ok ? ((u32)(8 * q) * row_bytes + (u32)(16 * c)) : kOutOfRange;
    bool row_ok[RG];
    u32 x_row[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        row_ok[r] = (m0 + 16 * r + c) < M;
        x_row[r] = (u32)(16 * r + c) * (u32)K * 2u;
    }
    // Whether this lane's eight K values of the slice's block ib exist.  The loop below is written with selects and
    // without exits between its parts: loads whose values are used in a later conditional block get moved
    // into that block by the compiler, next to their use, and then nothing is in flight ahead of the arithmetic.
    auto k_valid = [&](int ib) { return (ib < b_cnt) & ((b_beg + ib) * KB + 8 * q < K); };
    constexpr int CH = 2;  // K-blocks per wavefront and chunk (even: the W register sets alternate per block)

    f32x4 acc[RG][8], sum_acc[RG];
    float m_run[RG];  // running maximum of row c of each group over this wavefront's K-blocks so far
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        sum_acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run[r] = -__builtin_inff();
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto load_chunk = [&](u32x4 (&xs)[CH][RG], int i0) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int ib = i0 + u * NW;
#pragma unroll
            for (int r = 0; r < RG; ++r)
                xs[u][r] = load16(rx, (k_valid(ib) & row_ok[r]) ? x_row[r] + (u32)((b_beg + ib) * KB + 8 * q) * 2u : kOutOfRange);
        }
    };
    auto load_w = [&](WRows& w, int ib) {
        load_w_block(w, rw, (ib < b_cnt) ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange, row_bytes);
    };
    WRows w[2];
    auto chunk = [&](const u32x4 (&xs)[CH][RG], int i0) {
        float m_new[RG];
        bool moved = false;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            float cm = -__builtin_inff();
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const float mx = F::max8(xs[u][r]);
                cm = fmaxf(cm, (k_valid(i0 + u * NW) & row_ok[r]) ? mx : -__builtin_inff());
            }
            cm = fmaxf(cm, __shfl_xor(cm, 16, 64));
            cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
            m_new[r] = fmaxf(m_run[r], cm);
            moved |= (m_new[r] != m_run[r]);
        }
        if (__builtin_amdgcn_ballot_w64(moved) != 0) {
            // Accumulator element i of lane (q, c) belongs to row 4q + i; its factor lives in the lanes of row
            // 4q + i.  Rows that have seen nothing yet keep the factor 1 (their accumulators are zero).
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const float f = (m_run[r] == -__builtin_inff()) ? 1.0f
                                                               : __builtin_amdgcn_exp2f((m_run[r] - m_new[r]) * kLog2e);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float fi = __shfl(f, 4 * q + i, 64);
                    sum_acc[r][i] *= fi;
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[r][j][i] *= fi;
                }
                m_run[r] = m_new[r];
            }
        }
        float shift[RG];  // -max * log2(e): exp(x - max) = exp2(x * log2(e) + shift)
#pragma unroll
        for (int r = 0; r < RG; ++r) shift[r] = (m_run[r] != -__builtin_inff()) ? -m_run[r] * kLog2e : 0.f;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int ib = i0 + u * NW;                // a block past the end: its loads return zeros, a = 0
            load_w(w[(u + 1) & 1], ib + NW);           // the next block's W, into the other register set
            // The loads stay here, a whole block's arithmetic ahead of their use: without the fences the
            // scheduler pulls the next block's permutes up to just behind them.
            __builtin_amdgcn_sched_barrier(0);
            const bool kv = k_valid(ib);
            u32x4 a[RG];
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const bool v = kv & row_ok[r];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const float e0 = __builtin_amdgcn_exp2f(fmaf(F::lo(xs[u][r][d]), kLog2e, shift[r]));
                    const float e1 = __builtin_amdgcn_exp2f(fmaf(F::hi(xs[u][r][d]), kLog2e, shift[r]));
                    a[r][d] = v ? F::pack(e0, e1) : 0u;
                }
            }
            const WRows& wb = w[u & 1];
            auto step = [&](auto jc) {
                constexpr int J = decltype(jc)::value;
                const u32x4 b = b_operand<J>(wb);
#pragma unroll
                for (int r = 0; r < RG; ++r) acc[r][J] = F::mfma_16x16x32(a[r], b, acc[r][J]);
            };
            step(std::integral_constant<int, 0>{});
            step(std::integral_constant<int, 1>{});
            step(std::integral_constant<int, 2>{});
            step(std::integral_constant<int, 3>{});
            step(std::integral_constant<int, 4>{});
            step(std::integral_constant<int, 5>{});
            step(std::integral_constant<int, 6>{});
            step(std::integral_constant<int, 7>{});
            // The row sums ride on the matrix cores too: a ninth product against a block of ones adds up
            // exactly the rounded values the other eight use (every column of the result is the row sum).
#pragma unroll
            for (int r = 0; r < RG; ++r) sum_acc[r] = F::mfma_16x16x32(a[r], ones8<F>(), sum_acc[r]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    {
        u32x4 xa[CH][RG], xb[CH][RG];
        load_chunk(xa, wave);
        load_w(w[0], wave);
        // Two chunks per trip of the loop, no exit between them (a chunk past the end adds zeros).
        for (int i0 = wave; i0 < b_cnt; i0 += 2 * CH * NW) {
            load_chunk(xb, i0 + CH * NW);
            __builtin_amdgcn_sched_barrier(0);
            chunk(xa, i0);
            load_chunk(xa, i0 + 2 * CH * NW);
            __builtin_amdgcn_sched_barrier(0);
            chunk(xb, i0 + CH * NW);
        }
    }
#pragma unroll
    for (int r = 0; r < RG; ++r)
        if (q == 0) wave_max[wave * RB + 16 * r + c] = m_run[r];
    // Element i of the sum block in lane (q, c) is row 4q + i (any column: they are all equal).
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        if (c == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) wave_sum[wave * RB + 16 * r + 4 * q + i] = sum_acc[r][i];
        }
    }

    // ---- across wavefronts through LDS.  Accumulator j, element i of lane (q, c) is row 4q + i, column 8c + j.
    const int m = tid / TPR;
    const int col = (tid % TPR) * CPT;
    const int n = n0 + col;
#pragma unroll
    for (int r = 0; r < RG; ++r) store_acc_tile(red + r * kRedFloats + wave * 16 * TN, TN, q, c, acc[r]);
    __syncthreads();
    // Every wavefront's partials are relative to its own maximum: rescale to the workgroup's.
    float v[RG][CPT], den[RG], rmax[RG];
    bool out_ok[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        out_ok[r] = (m0 + 16 * r + m < M) && (n < N);  // N % 8 == 0 and CPT | 8: all CPT columns valid together
        den[r] = 0.f;
        rmax[r] = -__builtin_inff();
#pragma unroll
        for (int w8 = 0; w8 < NW; ++w8) rmax[r] = fmaxf(rmax[r], wave_max[w8 * RB + 16 * r + m]);
#pragma unroll
        for (int e = 0; e < CPT; ++e) v[r][e] = 0.f;
#pragma unroll
        for (int w8 = 0; w8 < NW; ++w8) {
            const float mw = wave_max[w8 * RB + 16 * r + m];
            // a wavefront without K-blocks (or a row past M) has maximum -inf and zero partials
            const float f = (mw == -__builtin_inff()) ? 0.f : __builtin_amdgcn_exp2f((mw - rmax[r]) * kLog2e);
            const float* src = red + r * kRedFloats + (w8 * 16 + m) * TN + col;
#pragma unroll
            for (int e = 0; e < CPT; ++e) v[r][e] = fmaf(f, src[e], v[r][e]);
            den[r] = fmaf(f, wave_sum[w8 * RB + 16 * r + m], den[r]);
        }
    }

    if (S > 1) {
        // Hand over (maximum, sum, partial product); the last arrival of the tile combines.
        const size_t tile_id = (size_t)rblock * n_tiles + ntile;
        float* ml = ml_part + (tile_id * S) * (2 * RB);
        const __amdgpu_buffer_rsrc_t racc = exchange_rsrc(acc_part, (size_t)S * M * N);
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            if (out_ok[r]) store_partial<CPT>(racc, acc_part, ((size_t)split * M + (m0 + 16 * r + m)) * N + n, v[r]);
            if (col == 0) store_coherent2(ml + (size_t)split * (2 * RB) + 2 * (16 * r + m), rmax[r], den[r]);
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

        // One round trip for up to eight slices: the (maximum, sum) pairs of every slice (S is at most
        // kSoftmaxMaxSplits) and the partial products of the first eight are requested together; the scale factors
        // 2^((m_s - max) log2 e) are worked out while the products are on their way.  Added in slice order.
        constexpr int BATCH = 8;
        static_assert(kSoftmaxMaxSplits == 2 * BATCH, "two batches of partial products");
        float fac[kSoftmaxMaxSplits][RG], gmax[RG];
        f32x2 mls[kSoftmaxMaxSplits][RG];
#pragma unroll
        for (int s = 0; s < kSoftmaxMaxSplits; ++s)
#pragma unroll
            for (int r = 0; r < RG; ++r)
                mls[s][r] = load_coherent2(ml + (size_t)min(s, S - 1) * (2 * RB) + 2 * (16 * r + m));
        float pa[BATCH][RG][CPT];
        auto load_batch = [&](int s0) {
#pragma unroll
            for (int j = 0; j < BATCH; ++j)
#pragma unroll
                for (int r = 0; r < RG; ++r)
                    load_partial<CPT>(racc, acc_part,
                                      out_ok[r] ? ((size_t)min(s0 + j, S - 1) * M + (m0 + 16 * r + m)) * N + n : (size_t)0, pa[j][r]);
        };
        auto add_batch = [&](int s0) {
#pragma unroll
            for (int j = 0; j < BATCH; ++j)
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const float f = fac[s0 + j][r];  // zero past the last slice and for a row or column past the end
#pragma unroll
                    for (int e = 0; e < CPT; ++e) v[r][e] = fmaf(f, pa[j][r][e], v[r][e]);
                }
        };
        load_batch(0);
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            gmax[r] = -__builtin_inff();
#pragma unroll
            for (int s = 0; s < kSoftmaxMaxSplits; ++s) gmax[r] = fmaxf(gmax[r], mls[s][r][0]);
            den[r] = 0.f;
#pragma unroll
            for (int s = 0; s < kSoftmaxMaxSplits; ++s) {
                fac[s][r] = (s < S && out_ok[r]) ? __builtin_amdgcn_exp2f((mls[s][r][0] - gmax[r]) * kLog2e) : 0.f;
                den[r] = fmaf(fac[s][r], mls[s][r][1], den[r]);
            }
#pragma unroll
            for (int e = 0; e < CPT; ++e) v[r][e] = 0.f;
        }
        add_batch(0);
        if (S > BATCH) {
            load_batch(BATCH);
            add_batch(BATCH);
        }
    }

    // The division after the loop (Figure 1(b)).
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        if (!out_ok[r]) continue;
        const float inv = 1.0f / den[r];
        *(u32x2*)(Y + (size_t)(m0 + 16 * r + m) * N + n) =
            u32x2{F::pack(v[r][0] * inv, v[r][1] * inv), F::pack(v[r][2] * inv, v[r][3] * inv)};
    }
}

template <typename F>
static hipError_t launch_split(const SoftmaxCall& c, int S, const SoftmaxWorkspace& ws) {
    dim3 grid((c.N + TN - 1) / TN, S, (c.M + RB - 1) / RB), block(NT);
    const size_t lds = (size_t)(RG * kRedFloats + 2 * NW * RB) * sizeof(float);
    auto kern = softmax_split_kernel<F>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c.stream, (const uint16_t*)c.X, (const uint16_t*)c.W, (uint16_t*)c.Y,
                       ws.acc_part, ws.ml_part, ws.tickets, c.M, c.K, c.N, S);
    return hipGetLastError();
}

hipError_t launch_softmax_split_16bit(const SoftmaxCall& c, bool f16, int split_k, const SoftmaxWorkspace& ws) {
    if (split_k < 1 || split_k > kSoftmaxMaxSplits) return hipErrorInvalidValue;
    return f16 ? launch_split<F16>(c, split_k, ws) : launch_split<Bf16>(c, split_k, ws);
}

}  // namespace prism
