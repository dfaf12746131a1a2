// Softmax followed by a matrix product with K split across workgroups (paper Figure 1; Table 1,
// "parallelized matmul (reduction)" and the compound parallelized sums).
//
// The kernel that gives a workgroup 16 rows over the whole of K makes every workgroup read all of its
// 128 columns of W: at the paper's shape (X[4096,4096], W[4096,128]) that is 1 MiB of W per 128 KiB of X,
// and the L2 -> CU path, not HBM, sets the time.  Here a workgroup owns 32 rows, 128 columns and one
// K-slice: half the W per row at once, and a further 1/S of it with S slices, while row blocks x slices
// still fill the chip.  The softmax of a slice is taken against the slice's own row maximum; what a
// workgroup hands over is (maximum, sum of exponentials, partial product), and the last arrival of a tile
// (atomic ticket) rescales every slice to the common maximum, adds them in slice order and divides: the
// same algebra as the division after the loop in Figure 1(b), applied once more across slices.
// When a wavefront's share of the slice is at most eight 32-deep K-blocks its part of X stays in
// registers between the maximum pass and the exponential pass: X is read exactly once.
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
constexpr int KEEP = kSoftmaxKeepBlocks;  // K-blocks of X a wavefront can hold in registers
constexpr int CPT = 16 * TN / NT;  // 4 columns per thread in the epilogue
constexpr int TPR = TN / CPT;      // 32 threads per output row
constexpr int kRedFloats = NW * 16 * TN;
constexpr float kLog2e = 1.4426950408889634f;

}  // namespace

template <typename F, bool RESIDENT>
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
    // Byte offset into X of this lane's 8 values of K-block ib of the slice, or "out of range" (reads as zero).
    auto x_off = [&](int ib, int r) -> u32 {
        const int k = (b_beg + ib) * KB + 8 * q;
        return (ib < b_cnt && k < K && row_ok[r]) ? x_row[r] + (u32)k * 2u : kOutOfRange;
    };
    auto k_valid = [&](int ib) { return ib < b_cnt && (b_beg + ib) * KB + 8 * q < K; };

    // ---- pass 1: the slice's row maxima.  All loads of a wavefront's share are issued before the first is
    // looked at: this pass pulls X from HBM.
    float mx[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) mx[r] = -__builtin_inff();
    u32x4 xk[RESIDENT ? KEEP : 1][RG];
    if (RESIDENT) {
#pragma unroll
        for (int u = 0; u < KEEP; ++u)
#pragma unroll
            for (int r = 0; r < RG; ++r) xk[u][r] = load16(rx, x_off(wave + u * NW, r));
#pragma unroll
        for (int u = 0; u < KEEP; ++u)
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const bool v = k_valid(wave + u * NW) && row_ok[r];
                mx[r] = fmaxf(mx[r], v ? F::max8(xk[u][r]) : -__builtin_inff());
            }
    } else {
        constexpr int U = 8;
        for (int i = wave; i < b_cnt; i += U * NW) {
            u32x4 xr[U][RG];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < RG; ++r) xr[u][r] = load16(rx, x_off(i + u * NW, r));
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const bool v = k_valid(i + u * NW) && row_ok[r];
                    mx[r] = fmaxf(mx[r], v ? F::max8(xr[u][r]) : -__builtin_inff());
                }
        }
    }
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        mx[r] = fmaxf(mx[r], __shfl_xor(mx[r], 16, 64));
        mx[r] = fmaxf(mx[r], __shfl_xor(mx[r], 32, 64));
        if (q == 0) wave_max[wave * RB + 16 * r + c] = mx[r];
    }
    __syncthreads();
    float shift[RG];  // -max * log2(e): exp(x - max) = exp2(x * log2(e) + shift)
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        float m = -__builtin_inff();
#pragma unroll
        for (int w = 0; w < NW; ++w) m = fmaxf(m, wave_max[w * RB + 16 * r + c]);
        shift[r] = row_ok[r] ? -m * kLog2e : 0.f;  // a row past M has no maximum: keep the arithmetic finite
    }

    // ---- pass 2: exp, row sums (a ninth MFMA against ones) and the product
    f32x4 acc[RG][8], sum_acc[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        sum_acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto load_w = [&](WRows& w, int ib) {
        load_w_block(w, rw, (ib < b_cnt) ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange, row_bytes);
    };
    auto consume = [&](const u32x4 (&xs)[RG], const WRows& w, int ib) {
        const bool kv = k_valid(ib);
        u32x4 a[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const bool v = kv && row_ok[r];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float e0 = __builtin_amdgcn_exp2f(fmaf(F::lo(xs[r][d]), kLog2e, shift[r]));
                const float e1 = __builtin_amdgcn_exp2f(fmaf(F::hi(xs[r][d]), kLog2e, shift[r]));
                a[r][d] = v ? F::pack(e0, e1) : 0u;
            }
        }
        auto step = [&](auto jc) {
            constexpr int J = decltype(jc)::value;
            const u32x4 b = b_operand<J>(w);
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
#pragma unroll
        for (int r = 0; r < RG; ++r) sum_acc[r] = F::mfma_16x16x32(a[r], ones8<F>(), sum_acc[r]);
    };
    if (RESIDENT) {
        // X is in registers; W blocks alternate between two register sets, the next one in flight.
        WRows w[2];
        load_w(w[0], wave);
#pragma unroll
        for (int u = 0; u < KEEP; ++u) {
            const int ib = wave + u * NW;
            if (ib < b_cnt) {  // uniform over the wavefront
                if (u + 1 < KEEP) load_w(w[(u + 1) & 1], ib + NW);
                consume(xk[u], w[u & 1], ib);
            }
        }
    } else {
        struct Trip {
            WRows w;
            u32x4 xr[RG];
        };
        auto issue = [&](Trip& t, int ib) {
#pragma unroll
            for (int r = 0; r < RG; ++r) t.xr[r] = load16(rx, x_off(ib, r));
            load_w(t.w, ib);
        };
        Trip ta, tb;
        int i = wave;
        if (i < b_cnt) {
            issue(ta, i);
            for (;;) {
                issue(tb, i + NW);
                consume(ta.xr, ta.w, i);
                i += NW;
                if (i >= b_cnt) break;
                issue(ta, i + NW);
                consume(tb.xr, tb.w, i);
                i += NW;
                if (i >= b_cnt) break;
            }
        }
    }
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
    float v[RG][CPT], den[RG], rmax[RG];
    bool out_ok[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        out_ok[r] = (m0 + 16 * r + m < M) && (n < N);  // N % 8 == 0 and CPT | 8: all CPT columns valid together
        den[r] = 0.f;
        rmax[r] = -__builtin_inff();
#pragma unroll
        for (int e = 0; e < CPT; ++e) v[r][e] = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float* src = red + r * kRedFloats + (w * 16 + m) * TN + col;
#pragma unroll
            for (int e = 0; e < CPT; ++e) v[r][e] += src[e];
            den[r] += wave_sum[w * RB + 16 * r + m];
            rmax[r] = fmaxf(rmax[r], wave_max[w * RB + 16 * r + m]);
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

        // Scale factors 2^((m_s - max) log2 e) of every slice first (S is at most kSoftmaxMaxSplits), then the
        // partial products four slices at a time, added in slice order.
        float fac[kSoftmaxMaxSplits][RG], gmax[RG];
        {
            f32x2 mls[kSoftmaxMaxSplits][RG];
#pragma unroll
            for (int s = 0; s < kSoftmaxMaxSplits; ++s)
#pragma unroll
                for (int r = 0; r < RG; ++r)
                    mls[s][r] = load_coherent2(ml + (size_t)min(s, S - 1) * (2 * RB) + 2 * (16 * r + m));
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
        }
        constexpr int BATCH = 4;
#pragma unroll
        for (int s0 = 0; s0 < kSoftmaxMaxSplits; s0 += BATCH) {
            if (s0 >= S) break;
            float pa[BATCH][RG][CPT];
#pragma unroll
            for (int j = 0; j < BATCH; ++j)
#pragma unroll
                for (int r = 0; r < RG; ++r)
                    if (out_ok[r])
                        load_partial<CPT>(racc, acc_part, ((size_t)min(s0 + j, S - 1) * M + (m0 + 16 * r + m)) * N + n, pa[j][r]);
#pragma unroll
            for (int j = 0; j < BATCH; ++j)
#pragma unroll
                for (int r = 0; r < RG; ++r)
                    if (out_ok[r]) {
                        const float f = fac[s0 + j][r];  // zero past the last slice
#pragma unroll
                        for (int e = 0; e < CPT; ++e) v[r][e] = fmaf(f, pa[j][r][e], v[r][e]);
                    }
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

template <typename F, bool RESIDENT>
static hipError_t launch_split(const SoftmaxCall& c, int S, const SoftmaxWorkspace& ws) {
    dim3 grid((c.N + TN - 1) / TN, S, (c.M + RB - 1) / RB), block(NT);
    const size_t lds = (size_t)(RG * kRedFloats + 2 * NW * RB) * sizeof(float);
    auto kern = softmax_split_kernel<F, RESIDENT>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c.stream, (const uint16_t*)c.X, (const uint16_t*)c.W, (uint16_t*)c.Y,
                       ws.acc_part, ws.ml_part, ws.tickets, c.M, c.K, c.N, S);
    return hipGetLastError();
}

hipError_t launch_softmax_split_16bit(const SoftmaxCall& c, bool f16, int split_k, const SoftmaxWorkspace& ws) {
    if (split_k < 1 || split_k > kSoftmaxMaxSplits) return hipErrorInvalidValue;
    const int kblocks = (c.K + KB - 1) / KB;
    const int per_wave = ((kblocks + split_k - 1) / split_k + NW - 1) / NW;
    const bool resident = per_wave <= KEEP;
    if (f16) return resident ? launch_split<F16, true>(c, split_k, ws) : launch_split<F16, false>(c, split_k, ws);
    return resident ? launch_split<Bf16, true>(c, split_k, ws) : launch_split<Bf16, false>(c, split_k, ws);
}

}  // namespace prism
