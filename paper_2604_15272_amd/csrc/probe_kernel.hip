// Probes for measurement (declared in prism_diag.h, not part of the operator boundary).
// Read-only probe: streams one or two [K, N] 16-bit matrices with the decode kernel's access pattern (a workgroup
// owns 128 columns and one K-slice; a wavefront's load covers 4 rows x 256 contiguous bytes, sixteen
// 16-byte row loads in flight per lane, non-temporal) and does nothing else.  Its time is what streaming W
// costs on the machine at hand: the floor the decode kernels are measured against.
#include "device_utils.h"
#include "prism_internal.h"

namespace prism {

template <bool TWO>
__global__ __launch_bounds__(512) void probe_stream_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ W2,
                                                           unsigned* __restrict__ sink, int K, int N, int S) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int n0 = blockIdx.x * kDecodeTileN, split = blockIdx.y;
    const int kblocks = (K + kDecodeKBlock - 1) / kDecodeKBlock;
    const int per = kblocks / S, rem = kblocks % S;
    const int b_beg = split * per + min(split, rem);
    const int b_cnt = per + (split < rem ? 1 : 0);
    const u32 row_bytes = (u32)N * 2u;
    const size_t w_first = (size_t)b_beg * kDecodeKBlock * N + n0;
    const size_t w_total = (size_t)K * N;
    const size_t w_left = (w_first < w_total ? w_total - w_first : 0) * 2;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(W + w_first, (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull));
    const __amdgpu_buffer_rsrc_t rw2 = make_rsrc((TWO ? W2 : W) + w_first, (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull));
    const u32 w_lane = (n0 + 8 * c) < N ? ((u32)(8 * q) * row_bytes + (u32)(16 * c)) : kOutOfRange;
    u32x4 acc = {0u, 0u, 0u, 0u};
    // As in the decode kernel: two K-blocks of one matrix per trip, or one K-block of each of two matrices.
    constexpr int U = 2, NW = 8;
    for (int i = wave; i < b_cnt; i += (TWO ? 1 : U) * NW) {
        u32x4 v[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int ib = TWO ? i : i + u * NW;
            const u32 off = ib < b_cnt ? w_lane + (u32)ib * kDecodeKBlock * row_bytes : kOutOfRange;
#pragma unroll
            for (int r = 0; r < 8; ++r) v[u][r] = load16_stream((TWO && u == 1) ? rw2 : rw, off + (u32)r * row_bytes);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < 8; ++r) acc ^= v[u][r];
    }
    // Keeps the loads alive; a matrix whose words fold to this value writes one word it may as well write.
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = 1u;
}

// The sixteen 128-byte address units of every 2 KiB, all read at the same time: workgroup j streams unit j % 16 of
// the 2 KiB blocks of its group (j / 16) - lanes 8 i .. 8 i + 7 read one 128-byte piece, consecutive pieces are 2 KiB
// apart, which is what a stripe of a matrix whose row pitch is a multiple of 2 KiB looks like to the memory system -
// with eight non-temporal 16-byte loads in flight per lane, and reports how long that took on the 100 MHz
// real-time counter.  Units that stream slowly while the others are busy too show up as longer times.
__global__ __launch_bounds__(512) void probe_units_kernel(const unsigned char* __restrict__ base, unsigned blocks_per_group,
                                                          unsigned long long* __restrict__ ticks) {
    const unsigned j = blockIdx.x, unit = j & 15u, group = j >> 4;
    const unsigned piece = threadIdx.x >> 3, sub = threadIdx.x & 7u;
    const __amdgpu_buffer_rsrc_t r =
        make_rsrc(base + (size_t)group * blocks_per_group * 2048u, blocks_per_group * 2048u);  // below 2 GiB (host)
    const unsigned long long t0 = wall_clock64();
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (unsigned b = piece; b < blocks_per_group; b += 8u * 64u) {
        u32x4 v[8];
#pragma unroll
        for (unsigned i = 0; i < 8; ++i) {
            const unsigned bb = b + i * 64u;
            v[i] = load16_stream(r, bb < blocks_per_group ? bb * 2048u + unit * 128u + sub * 16u : kOutOfRange);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc ^= v[i];
    }
    // the value is consumed before the clock is read again: the loads have landed
    const unsigned fold = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    __syncthreads();
    if (threadIdx.x == 0) ticks[j] = wall_clock64() - t0 + (fold == 0x9E3779B9u ? 1u : 0u);
}

hipError_t launch_probe_units(const void* base, unsigned blocks_per_group, int groups, unsigned long long* ticks,
                              hipStream_t stream) {
    hipLaunchKernelGGL(probe_units_kernel, dim3(16 * groups), dim3(512), 0, stream, (const unsigned char*)base,
                       blocks_per_group, ticks);
    return hipGetLastError();
}

// What one compute unit's vector-memory path delivers for a given shape of load instruction, on data that stays in
// the L2: every workgroup (eight wavefronts, eight loads in flight per lane) reads the same 1 MiB region `reps`
// times and computes nothing; ticks[8 j + w] receives the shader clock cycles wavefront w of workgroup j needed.
// The region is 128 rows of 8 KiB; a "block" is eight load instructions = 8 KiB (4 KiB for pattern 3), 128 blocks.
//   0: four rows x 256 contiguous bytes per instruction (how the decode kernels read W)
//   1: sixteen rows x 64 bytes per instruction (an X operand in MFMA layout: lane (q, c) = row c, eight K values)
//   2: eight rows x 128 bytes per instruction (how the prefill kernel requests X)
//   3: four rows x 128 bytes per instruction with 8-byte loads
template <int PATTERN>
__global__ __launch_bounds__(512) void probe_loads_kernel(const unsigned char* __restrict__ base, int reps,
                                                          unsigned long long* __restrict__ ticks) {
    constexpr u32 kPitch = 8192;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u32 q = lane >> 4, c = lane & 15;
    const __amdgpu_buffer_rsrc_t r = make_rsrc(base, 128u * kPitch);  // the host checked that the buffer holds it
    u32 acc = 0;
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int rep = 0; rep < reps; ++rep) {
        for (u32 ib = wave; ib < 128; ib += 8) {
            if constexpr (PATTERN == 3) {
                u32x2 v[8];
#pragma unroll
                for (u32 i = 0; i < 8; ++i)
                    v[i] = __builtin_amdgcn_raw_buffer_load_b64(r, (int)((4 * i + q + 32 * (ib & 3)) * kPitch + (ib >> 2) * 128 + 8 * c), 0, 0);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc ^= v[i][0] ^ v[i][1];
            } else {
                u32x4 v[8];
#pragma unroll
                for (u32 i = 0; i < 8; ++i) {
                    u32 off;
                    if (PATTERN == 0) off = (4 * i + q + 32 * (ib & 3)) * kPitch + (ib >> 2) * 256 + 16 * c;
                    else if (PATTERN == 1) off = (16 * i + c) * kPitch + (ib * 32 + 8 * q) * 2;
                    else off = (8 * i + (lane >> 3) + 64 * (ib & 1)) * kPitch + (ib >> 1) * 128 + 16 * (lane & 7);
                    v[i] = load16(r, off);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) acc ^= v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
            }
        }
    }
    // the values are consumed before the clock is read again: the loads have landed
    const unsigned long long t1 = __builtin_readcyclecounter() + (acc == 0x9E3779B9u ? 1u : 0u);
    if (lane == 0) ticks[blockIdx.x * 8 + wave] = t1 - t0;
}

hipError_t launch_probe_loads(const void* base, int pattern, int reps, int workgroups, unsigned long long* ticks,
                              hipStream_t stream) {
    const unsigned char* b = (const unsigned char*)base;
    if (pattern == 0) hipLaunchKernelGGL(probe_loads_kernel<0>, dim3(workgroups), dim3(512), 0, stream, b, reps, ticks);
    else if (pattern == 1) hipLaunchKernelGGL(probe_loads_kernel<1>, dim3(workgroups), dim3(512), 0, stream, b, reps, ticks);
    else if (pattern == 2) hipLaunchKernelGGL(probe_loads_kernel<2>, dim3(workgroups), dim3(512), 0, stream, b, reps, ticks);
    else if (pattern == 3) hipLaunchKernelGGL(probe_loads_kernel<3>, dim3(workgroups), dim3(512), 0, stream, b, reps, ticks);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// A buffer read front to back: workgroup j streams the j-th of gridDim.x equal contiguous pieces (every wavefront
// instruction covers 1 KiB of consecutive bytes, sixteen 16-byte loads in flight per lane, non-temporal).  The
// simplest access pattern there is: what the same bytes cost when no stripe structure is imposed on them.
__global__ __launch_bounds__(512) void probe_linear_kernel(const unsigned char* __restrict__ base, unsigned long long bytes,
                                                           unsigned* __restrict__ sink) {
    const unsigned long long per = (bytes / gridDim.x) & ~1023ull;
    const unsigned long long first = per * blockIdx.x;
    const unsigned long long len = blockIdx.x + 1 == gridDim.x ? bytes - first : per;
    const __amdgpu_buffer_rsrc_t r = make_rsrc(base + first, (u32)(len < 0x7FFFFFFFull ? len : 0x7FFFFFFFull));
    u32x4 acc = {0u, 0u, 0u, 0u};
    constexpr unsigned kStep = 512 * 16;  // bytes the workgroup covers with one load per thread
    for (unsigned long long off = 0; off < len; off += 16ull * kStep) {
        u32x4 v[16];
#pragma unroll
        for (unsigned i = 0; i < 16; ++i) {
            const unsigned long long o = off + (unsigned long long)i * kStep + threadIdx.x * 16u;
            v[i] = load16_stream(r, o < len ? (u32)o : kOutOfRange);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) acc ^= v[i];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = 1u;
}

hipError_t launch_probe_linear(const void* base, unsigned long long bytes, int workgroups, unsigned* sink, hipStream_t stream) {
    hipLaunchKernelGGL(probe_linear_kernel, dim3(workgroups), dim3(512), 0, stream, (const unsigned char*)base, bytes, sink);
    return hipGetLastError();
}

// Matrix pipes alone: every wavefront (four per workgroup, one per SIMD) issues 16 x iters independent-enough
// 32x32x16 bf16 MFMAs on registers; no memory, no LDS.  What the part sustains under its power limit.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    const u32 lane = threadIdx.x & 63;
    const u32x4 a = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    const u32x4 b = {0x3C003C00u + lane, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = Bf16::mfma_32x32x16(a, b, acc[j]);
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += acc[j][v];
    if (t == -1.0f) sink[0] = t;  // never true (the sums are positive): keeps the MFMAs alive
}

hipError_t launch_probe_mfma(float* sink, int workgroups, int iters, hipStream_t stream) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, stream, sink, iters);
    return hipGetLastError();
}

hipError_t launch_probe_stream(const void* W, const void* W2, unsigned* sink, int K, int N, int S, hipStream_t stream) {
    dim3 grid((N + kDecodeTileN - 1) / kDecodeTileN, S), block(512);
    if (W2)
        hipLaunchKernelGGL(probe_stream_kernel<true>, grid, block, 0, stream, (const uint16_t*)W, (const uint16_t*)W2, sink,
                           K, N, S);
    else
        hipLaunchKernelGGL(probe_stream_kernel<false>, grid, block, 0, stream, (const uint16_t*)W, (const uint16_t*)W, sink,
                           K, N, S);
    return hipGetLastError();
}

}  // namespace prism
