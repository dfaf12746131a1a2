// Softmax followed by a matrix product, Y = softmax(X over k) . W: the paper's running example
// (Figure 1).  The fused program of Figure 1(b) keeps two accumulators in its loop over k, the row
// sum of exp(X) and the product exp(X) . W, and divides after the loop; softmax(X) is never written
// to memory.  Both kernels here have that structure.  What the figure leaves out and a library
// needs is the row maximum: exp(x - max) instead of exp(x), which changes nothing in exact
// arithmetic and keeps every term in (0, 1].  The matrix-core kernel keeps a running maximum per wavefront
// and rescales its accumulators when it moves (so X is read once, streaming under the arithmetic); the plain
// kernel finds the maximum in a first pass over the same rows.
//
// Matrix-core kernel (16-bit storage): a workgroup owns 16 rows (one MFMA row group) and 128 columns
// of W; its wavefronts take the 32-deep K-blocks round-robin.  X is K-contiguous, which is the
// layout of an MFMA A operand, so a lane loads its 8 K values of a row straight from memory,
// applies exp and rounds to the storage format; the row sums are a ninth MFMA against ones, so
// numerator and denominator weigh the same rounded values.  W is handled as in the decode kernel (8 x 8 sub-blocks per lane,
// permuted into B operands).  The partial products, sums and maxima of the wavefronts meet in LDS.
// X is the large operand here and the roofline is streaming it from HBM once; what the kernel is
// actually bound by at the paper's shape is the vector pipe (exponentials, conversions, the permutes
// of W, which every workgroup re-reads from the L2 for its 16 rows).
//
// Plain kernel: any shape and storage type, 8 rows x 256 columns per workgroup, fp32 arithmetic.
#include <type_traits>

#include "device_utils.h"
#include "prism_internal.h"
#include "w_block.h"

namespace prism {

namespace {

constexpr int TN = 128;  // columns of W per workgroup (matrix-core kernel)
constexpr int KB = 32;   // K depth of one MFMA

template <typename T> __device__ __forceinline__ float ld_elem(const T* p, size_t i);
template <> __device__ __forceinline__ float ld_elem<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld_elem<uint16_t>(const uint16_t* p, size_t i) {
    return __builtin_bit_cast(float, (u32)p[i] << 16);
}
template <> __device__ __forceinline__ float ld_elem<_Float16>(const _Float16* p, size_t i) { return (float)p[i]; }
template <typename T> __device__ __forceinline__ void st_elem(T* p, size_t i, float v);
template <> __device__ __forceinline__ void st_elem<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st_elem<uint16_t>(uint16_t* p, size_t i, float v) {
    p[i] = (uint16_t)(pack_bf16(v, 0.0f) & 0xFFFFu);
}
template <> __device__ __forceinline__ void st_elem<_Float16>(_Float16* p, size_t i, float v) { p[i] = (_Float16)v; }

}  // namespace

// ---- matrix-core kernel --------------------------------------------------------------------------
// A wavefront walks its K-blocks in chunks of CH.  Per chunk: the chunk's row maxima (from the registers
// the loads landed in), the running maximum, a rescale of the accumulators by 2^((old - new) log2 e) if
// it moved, then exp, row sums and products of the chunk's K-blocks.  The next chunk's X is requested
// before the current one is worked on, so the stream from HBM runs under the arithmetic.
template <typename F, int NW>
__global__ __launch_bounds__(NW * 64) void softmax_rows_kernel(const uint16_t* __restrict__ X,
                                                               const uint16_t* __restrict__ W,
                                                               uint16_t* __restrict__ Y, int M, int K, int N) {
    constexpr int NT = NW * 64;
    constexpr int CPT = 16 * TN / NT;  // columns per thread in the epilogue
    constexpr int TPR = TN / CPT;      // threads per output row
    static_assert(CPT == 2 || CPT == 4 || CPT == 8, "epilogue mapping");
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr int CH = 4;  // K-blocks per wavefront and chunk (even: the W register sets alternate per block)

    extern __shared__ __align__(16) float lds[];  // 16-byte LDS accesses need the alignment said
    float* red = lds;                       // [NW][16][TN]
    float* wave_max = lds + NW * 16 * TN;   // [NW][16]
    float* wave_sum = wave_max + NW * 16;   // [NW][16]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int n0 = blockIdx.x * TN, m0 = blockIdx.y * 16;
    const int kblocks = (K + KB - 1) / KB;

    // Descriptors: X from this workgroup's first row to the end of the matrix (rows past M are masked),
    // W from its first column to the end.
    const size_t x_left = ((size_t)(M - m0) * K) * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + (size_t)m0 * K, (u32)(x_left < 0x7FFFFFFFull ? x_left : 0x7FFFFFFFull));
    const size_t w_left = ((size_t)K * N - n0) * 2;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(W + n0, (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull));
    const u32 row_bytes = (u32)N * 2u;
    const bool col_ok = (n0 + 8 * c) < N;
    const u32 w_lane = col_ok ? ((u32)(8 * q) * row_bytes + (u32)(16 * c)) : kOutOfRange;
    const bool row_ok = (m0 + c) < M;
    const u32 x_row = (u32)c * (u32)K * 2u;
    // Whether this lane's eight K values of block ib exist (implies ib < kblocks).  Everything in the loop below is
    // written with selects, not branches: loads whose values are used in a later conditional block get moved
    // into that block by the compiler, next to their use, and then nothing is in flight ahead of the arithmetic.
    auto k_valid = [&](int ib) { return ib * KB + 8 * q < K; };

    f32x4 acc[8], sum_acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -__builtin_inff();  // running maximum of row c over this wavefront's K-blocks so far

    auto load_chunk = [&](u32x4 (&xs)[CH], int i0) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int ib = i0 + u * NW;
            xs[u] = load16(rx, (k_valid(ib) & row_ok) ? x_row + (u32)(ib * KB + 8 * q) * 2u : kOutOfRange);
        }
    };
    auto load_w = [&](WRows& w, int ib) {
        load_w_block(w, rw, (ib < kblocks) ? w_lane + (u32)ib * KB * row_bytes : kOutOfRange, row_bytes);
    };
    WRows w[2];
    auto chunk = [&](const u32x4 (&xs)[CH], int i0) {
        float cm = -__builtin_inff();
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const float mx = F::max8(xs[u]);
            cm = fmaxf(cm, (k_valid(i0 + u * NW) & row_ok) ? mx : -__builtin_inff());
        }
        cm = fmaxf(cm, __shfl_xor(cm, 16, 64));
        cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
        const float m_new = fmaxf(m_run, cm);
        if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
            // Accumulator element i of lane (q, c) belongs to row 4q + i; its factor lives in the lanes of row
            // 4q + i.  Rows that have seen nothing yet keep the factor 1 (their accumulators are zero).
            const float f = (m_run == -__builtin_inff()) ? 1.0f : __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float fi = __shfl(f, 4 * q + i, 64);
                sum_acc[i] *= fi;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j][i] *= fi;
            }
            m_run = m_new;
        }
        const float shift = row_ok ? -m_run * kLog2e : 0.f;  // a row past M has no maximum: keep the arithmetic finite
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int ib = i0 + u * NW;                // a block past the end: its loads return zeros, a = 0
            load_w(w[(u + 1) & 1], ib + NW);           // the next block's W, into the other register set
            // The loads stay here, a whole block's arithmetic ahead of their use: without the fences the
            // scheduler pulls the next block's permutes up to just behind them.
            __builtin_amdgcn_sched_barrier(0);
            const bool v = k_valid(ib) & row_ok;
            u32x4 a;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float e0 = __builtin_amdgcn_exp2f(fmaf(F::lo(xs[u][d]), kLog2e, shift));
                const float e1 = __builtin_amdgcn_exp2f(fmaf(F::hi(xs[u][d]), kLog2e, shift));
                a[d] = v ? F::pack(e0, e1) : 0u;
            }
            const WRows& wb = w[u & 1];
            acc[0] = F::mfma_16x16x32(a, b_operand<0>(wb), acc[0]);
            acc[1] = F::mfma_16x16x32(a, b_operand<1>(wb), acc[1]);
            acc[2] = F::mfma_16x16x32(a, b_operand<2>(wb), acc[2]);
            acc[3] = F::mfma_16x16x32(a, b_operand<3>(wb), acc[3]);
            acc[4] = F::mfma_16x16x32(a, b_operand<4>(wb), acc[4]);
            acc[5] = F::mfma_16x16x32(a, b_operand<5>(wb), acc[5]);
            acc[6] = F::mfma_16x16x32(a, b_operand<6>(wb), acc[6]);
            acc[7] = F::mfma_16x16x32(a, b_operand<7>(wb), acc[7]);
            // The row sums ride on the matrix cores too: a ninth product against a block of ones adds up
            // exactly the rounded values the other eight use (every column of the result is the row sum).
            sum_acc = F::mfma_16x16x32(a, ones8<F>(), sum_acc);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    {
        u32x4 xa[CH], xb[CH];
        load_chunk(xa, wave);
        load_w(w[0], wave);
        // Two chunks per trip of the loop, no exit between them (a chunk past the end adds zeros): see k_valid.
        for (int i0 = wave; i0 < kblocks; i0 += 2 * CH * NW) {
            load_chunk(xb, i0 + CH * NW);
            __builtin_amdgcn_sched_barrier(0);
            chunk(xa, i0);
            load_chunk(xa, i0 + 2 * CH * NW);
            __builtin_amdgcn_sched_barrier(0);
            chunk(xb, i0 + CH * NW);
        }
    }
    // Element i of the sum block in lane (q, c) is row 4q + i (any column c: they are all equal).
    if (c == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) wave_sum[wave * 16 + 4 * q + i] = sum_acc[i];
    }
    if (q == 0) wave_max[wave * 16 + c] = m_run;

    // ---- across wavefronts through LDS: every wavefront's partials are relative to its own maximum, so they
    // are rescaled to the common one; then the division (Figure 1(b): Div after the loop).
    // Accumulator j, element i of lane (q, c) is row 4q + i, column 8c + j.
    const int m = tid / TPR;
    const int col = (tid % TPR) * CPT;
    const int n = n0 + col;
    store_acc_tile(red + wave * 16 * TN, TN, q, c, acc);
    __syncthreads();
    float gmax = -__builtin_inff();
#pragma unroll
    for (int w8 = 0; w8 < NW; ++w8) gmax = fmaxf(gmax, wave_max[w8 * 16 + m]);
    float v[CPT], den = 0.f;
#pragma unroll
    for (int e = 0; e < CPT; ++e) v[e] = 0.f;
#pragma unroll
    for (int w8 = 0; w8 < NW; ++w8) {
        const float mw = wave_max[w8 * 16 + m];
        // a wavefront without K-blocks (or a row past M) has maximum -inf and zero partials
        const float f = (mw == -__builtin_inff()) ? 0.f : __builtin_amdgcn_exp2f((mw - gmax) * kLog2e);
        const float* src = red + (w8 * 16 + m) * TN + col;
#pragma unroll
        for (int e = 0; e < CPT; ++e) v[e] = fmaf(f, src[e], v[e]);
        den = fmaf(f, wave_sum[w8 * 16 + m], den);
    }
    const int row = m0 + m;
    if (row < M && n < N) {  // N % 8 == 0 and CPT | 8: all CPT columns valid together
        const float inv = 1.0f / den;
        u32 packed[CPT / 2];
#pragma unroll
        for (int e = 0; e < CPT / 2; ++e) packed[e] = F::pack(v[2 * e] * inv, v[2 * e + 1] * inv);
        uint16_t* out = Y + (size_t)row * N + n;
        if (CPT == 2) *(u32*)out = packed[0];
        if (CPT == 4) *(u32x2*)out = u32x2{packed[0], packed[1]};
        if (CPT == 8) *(u32x4*)out = u32x4{packed[0], packed[1], packed[2 % (CPT / 2)], packed[3 % (CPT / 2)]};
    }
}

template <typename F>
static hipError_t launch_softmax_rows_fmt(const SoftmaxCall& c) {
    constexpr int NW = 8;
    dim3 grid((c.N + TN - 1) / TN, (c.M + 15) / 16), block(NW * 64);
    const size_t lds = (size_t)(NW * 16 * TN + 2 * NW * 16) * sizeof(float);
    auto kern = softmax_rows_kernel<F, NW>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c.stream, (const uint16_t*)c.X, (const uint16_t*)c.W, (uint16_t*)c.Y,
                       c.M, c.K, c.N);
    return hipGetLastError();
}

hipError_t launch_softmax_rows_16bit(const SoftmaxCall& c, bool f16) {
    return f16 ? launch_softmax_rows_fmt<F16>(c) : launch_softmax_rows_fmt<Bf16>(c);
}

// ---- plain kernel -----------------------------------------------------------------------------------
constexpr int kSmRows = 8;
constexpr int kSmCols = 256;

template <typename T>
__global__ __launch_bounds__(kSmCols) void softmax_simple_kernel(const T* __restrict__ X, const T* __restrict__ W,
                                                               T* __restrict__ Y, int M, int K, int N) {
    __shared__ float es[kSmRows][kSmCols];
    __shared__ float part[kSmCols / 64][kSmRows];
    __shared__ float row_max[kSmRows];
    const int t = threadIdx.x;
    const int n = blockIdx.x * kSmCols + t;
    const int m0 = blockIdx.y * kSmRows;
    const bool col_ok = n < N;

    // pass 1: row maxima (threads stride over k; lanes, then wavefronts)
    float mx[kSmRows];
#pragma unroll
    for (int r = 0; r < kSmRows; ++r) mx[r] = -__builtin_inff();
    for (int k = t; k < K; k += kSmCols) {
#pragma unroll
        for (int r = 0; r < kSmRows; ++r)
            if (m0 + r < M) mx[r] = fmaxf(mx[r], ld_elem<T>(X, (size_t)(m0 + r) * K + k));
    }
#pragma unroll
    for (int r = 0; r < kSmRows; ++r) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx[r] = fmaxf(mx[r], __shfl_xor(mx[r], off, 64));
    }
    if ((t & 63) == 0) {
#pragma unroll
        for (int r = 0; r < kSmRows; ++r) part[t >> 6][r] = mx[r];
    }
    __syncthreads();
    if (t < kSmRows) {
        float m = part[0][t];
#pragma unroll
        for (int w = 1; w < kSmCols / 64; ++w) m = fmaxf(m, part[w][t]);
        row_max[t] = (m0 + t < M) ? m : 0.f;
    }
    __syncthreads();

    // pass 2: exp and its row sum in the loop over k beside the product; the division after it
    float acc[kSmRows], sum[kSmRows];
#pragma unroll
    for (int r = 0; r < kSmRows; ++r) { acc[r] = 0.f; sum[r] = 0.f; }
    for (int kc = 0; kc < K; kc += kSmCols) {
        __syncthreads();
        const int k = kc + t;
#pragma unroll
        for (int r = 0; r < kSmRows; ++r) {
            const int m = m0 + r;
            const float e = (k < K && m < M) ? expf(ld_elem<T>(X, (size_t)m * K + k) - row_max[r]) : 0.f;
            sum[r] += e;
            es[r][t] = e;
        }
        __syncthreads();
        const int kend = min(kSmCols, K - kc);
        if (col_ok) {
            for (int kk = 0; kk < kend; ++kk) {
                const float w = ld_elem<T>(W, (size_t)(kc + kk) * N + n);
#pragma unroll
                for (int r = 0; r < kSmRows; ++r) acc[r] = fmaf(es[r][kk], w, acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kSmRows; ++r) {
        float v = sum[r];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        sum[r] = v;
    }
    __syncthreads();
    if ((t & 63) == 0) {
#pragma unroll
        for (int r = 0; r < kSmRows; ++r) part[t >> 6][r] = sum[r];
    }
    __syncthreads();
    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < kSmRows; ++r) {
        const int m = m0 + r;
        if (m >= M) break;
        float den = 0.f;
#pragma unroll
        for (int w = 0; w < kSmCols / 64; ++w) den += part[w][r];
        st_elem<T>(Y, (size_t)m * N + n, acc[r] / den);
    }
}

template <typename T>
static hipError_t launch_softmax_simple_t(const SoftmaxCall& c) {
    dim3 grid((c.N + kSmCols - 1) / kSmCols, (c.M + kSmRows - 1) / kSmRows), block(kSmCols);
    hipLaunchKernelGGL((softmax_simple_kernel<T>), grid, block, 0, c.stream, (const T*)c.X, (const T*)c.W, (T*)c.Y, c.M,
                       c.K, c.N);
    return hipGetLastError();
}

hipError_t launch_softmax_simple(const SoftmaxCall& c, int dtype) {
    if (dtype == PRISM_F32) return launch_softmax_simple_t<float>(c);
    if (dtype == PRISM_F16) return launch_softmax_simple_t<_Float16>(c);
    return launch_softmax_simple_t<uint16_t>(c);
}

}  // namespace prism
