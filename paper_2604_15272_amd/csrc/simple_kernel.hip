// Plain FMA kernel for any M, K, N and every storage type.
//
// One workgroup owns an 8-row by 256-column output tile.  It walks K in chunks: each chunk of X is
// staged in LDS already multiplied by the gain, while the raw squares are summed on the side
// (the row reduction lives in the K-loop, as in the paper's fused program of Figure 1(b)); every
// thread then runs the chunk against its own column of W.  1/rms goes on after the loop
// (Table 1, "matmul commutes with div denominator").
#include "device_utils.h"
#include "prism_internal.h"

namespace prism {

constexpr int kSimpleRows = 8;
constexpr int kSimpleCols = 256;
constexpr int kSimpleChunk = 256;

template <typename T> __device__ __forceinline__ float load_elem(const T* p, size_t i);
template <> __device__ __forceinline__ float load_elem<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t* p, size_t i) {
    return __builtin_bit_cast(float, (u32)p[i] << 16);
}
template <> __device__ __forceinline__ float load_elem<_Float16>(const _Float16* p, size_t i) { return (float)p[i]; }
template <typename T> __device__ __forceinline__ void store_elem(T* p, size_t i, float v);
template <> __device__ __forceinline__ void store_elem<_Float16>(_Float16* p, size_t i, float v) { p[i] = (_Float16)v; }
template <> __device__ __forceinline__ void store_elem<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_elem<uint16_t>(uint16_t* p, size_t i, float v) {
    p[i] = (uint16_t)(pack_bf16(v, 0.0f) & 0xFFFFu);
}

template <typename T, bool GATED>
__global__ __launch_bounds__(kSimpleCols) void simple_kernel(const T* __restrict__ X, const T* __restrict__ g,
                                                           const T* __restrict__ W1, const T* __restrict__ W2,
                                                           T* __restrict__ Y, int M, int K, int N, float eps, int flags) {
    __shared__ float xs[kSimpleRows][kSimpleChunk];
    __shared__ float ss_wave[kSimpleCols / 64][kSimpleRows];
    const int t = threadIdx.x;
    const int n = blockIdx.x * kSimpleCols + t;
    const int m0 = blockIdx.y * kSimpleRows;
    const bool col_ok = n < N;

    float acc1[kSimpleRows], acc2[kSimpleRows], ss[kSimpleRows];
#pragma unroll
    for (int r = 0; r < kSimpleRows; ++r) { acc1[r] = 0.f; acc2[r] = 0.f; ss[r] = 0.f; }

    for (int kc = 0; kc < K; kc += kSimpleChunk) {
        __syncthreads();
        const int k = kc + t;
        const float gk = (k < K) ? ((flags & kFlagGain) ? load_elem<T>(g, (size_t)k) : 1.f) : 0.f;
#pragma unroll
        for (int r = 0; r < kSimpleRows; ++r) {
            const int m = m0 + r;
            const float x = (k < K && m < M) ? load_elem<T>(X, (size_t)m * K + k) : 0.f;
            ss[r] = fmaf(x, x, ss[r]);
            xs[r][t] = x * gk;
        }
        __syncthreads();
        const int kend = min(kSimpleChunk, K - kc);
        if (col_ok) {
            for (int kk = 0; kk < kend; ++kk) {
                const size_t wi = (size_t)(kc + kk) * N + n;
                const float w1 = load_elem<T>(W1, wi);
                float w2 = 0.f;
                if (GATED) w2 = load_elem<T>(W2, wi);
#pragma unroll
                for (int r = 0; r < kSimpleRows; ++r) {
                    const float a = xs[r][kk];
                    acc1[r] = fmaf(a, w1, acc1[r]);
                    if (GATED) acc2[r] = fmaf(a, w2, acc2[r]);
                }
            }
        }
    }

    // Row sums of squares: across the 64 lanes of a wavefront, then across the wavefronts.
#pragma unroll
    for (int r = 0; r < kSimpleRows; ++r) {
        float v = ss[r];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        ss[r] = v;
    }
    if ((t & 63) == 0) {
#pragma unroll
        for (int r = 0; r < kSimpleRows; ++r) ss_wave[t >> 6][r] = ss[r];
    }
    __syncthreads();
    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < kSimpleRows; ++r) {
        const int m = m0 + r;
        if (m >= M) break;
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < kSimpleCols / 64; ++w) tot += ss_wave[w][r];
        const float rinv = (flags & kFlagNorm) ? 1.0f / sqrtf(tot / (float)K + eps) : 1.0f;
        float y = acc1[r] * rinv;
        if (GATED) {
            const float a = y;
            y = ((flags & kFlagSilu) ? a / (1.0f + expf(-a)) : a) * (acc2[r] * rinv);
        }
        store_elem<T>(Y, (size_t)m * N + n, y);
    }
}

template <typename T>
static hipError_t launch_simple(const Call& c) {
    dim3 grid((c.N + kSimpleCols - 1) / kSimpleCols, (c.M + kSimpleRows - 1) / kSimpleRows);
    dim3 block(kSimpleCols);
    if (c.gated)
        hipLaunchKernelGGL((simple_kernel<T, true>), grid, block, 0, c.stream, (const T*)c.X, (const T*)c.g,
                           (const T*)c.W1, (const T*)c.W2, (T*)c.Y, c.M, c.K, c.N, c.eps, c.flags);
    else
        hipLaunchKernelGGL((simple_kernel<T, false>), grid, block, 0, c.stream, (const T*)c.X, (const T*)c.g,
                           (const T*)c.W1, (const T*)c.W1, (T*)c.Y, c.M, c.K, c.N, c.eps, c.flags);
    return hipGetLastError();
}

hipError_t launch_simple_f32(const Call& c) { return launch_simple<float>(c); }
hipError_t launch_simple_bf16(const Call& c) { return launch_simple<uint16_t>(c); }
hipError_t launch_simple_f16(const Call& c) { return launch_simple<_Float16>(c); }

}  // namespace prism
