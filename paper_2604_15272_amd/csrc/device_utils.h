// Device-side helpers for gfx950: vector types, bf16 packing, buffer loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace prism {

typedef unsigned int u32;
typedef __attribute__((ext_vector_type(2))) u32 u32x2;
typedef __attribute__((ext_vector_type(3))) u32 u32x3;
typedef __attribute__((ext_vector_type(4))) u32 u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// A voffset no buffer of less than 2 GiB contains: loads from it return zero.
constexpr u32 kOutOfRange = 0x80000000u;

__device__ __forceinline__ float bf16_lo(u32 u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(u32 u) { return __builtin_bit_cast(float, u & 0xFFFF0000u); }

// Two floats -> two bf16 (round to nearest even) in one dword, a in the low half.
__device__ __forceinline__ u32 pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(u32, __builtin_convertvector(v, bf16x2));
}

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

// The two 16-bit storage formats of the matrix-core kernels.  A dword holds two elements, the one at
// the lower address in its low half.  lo/hi widen exactly to fp32; pack rounds two fp32 values to
// nearest even; the MFMA wrappers take operands as raw dwords.
struct Bf16 {
    static constexpr u32 kOnePair = 0x3F803F80u;  // two elements of value 1
    static __device__ __forceinline__ float lo(u32 u) { return bf16_lo(u); }
    static __device__ __forceinline__ float hi(u32 u) { return bf16_hi(u); }
    static __device__ __forceinline__ u32 pack(float a, float b) { return pack_bf16(a, b); }
    // Largest of the eight elements of four dwords.
    static __device__ __forceinline__ float max8(u32x4 x) {
        float v = lo(x[0]);
#pragma unroll
        for (int d = 0; d < 4; ++d) v = fmaxf(v, fmaxf(lo(x[d]), hi(x[d])));
        return v;
    }
    static __device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                       0, 0);
    }
    static __device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                       0, 0);
    }
};
struct F16 {
    static constexpr u32 kOnePair = 0x3C003C00u;
    static __device__ __forceinline__ float lo(u32 u) { return (float)__builtin_bit_cast(f16x2, u)[0]; }
    static __device__ __forceinline__ float hi(u32 u) { return (float)__builtin_bit_cast(f16x2, u)[1]; }
    static __device__ __forceinline__ u32 pack(float a, float b) {
        const f16x2 v = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(u32, v);
    }
    // Largest of the eight elements of four dwords: pairwise in the storage format (packed maximum), widened once.
    static __device__ __forceinline__ float max8(u32x4 x) {
        // The dwords are copied out first: a bit cast applied directly to an element of the vector reads element 0
        // whichever index is written (seen with this compiler), which made this the maximum of two values only.
        const u32 d0 = x[0], d1 = x[1], d2 = x[2], d3 = x[3];
        f16x2 m = __builtin_elementwise_max(__builtin_bit_cast(f16x2, d0), __builtin_bit_cast(f16x2, d1));
        m = __builtin_elementwise_max(m, __builtin_elementwise_max(__builtin_bit_cast(f16x2, d2), __builtin_bit_cast(f16x2, d3)));
        return fmaxf((float)m[0], (float)m[1]);
    }
    static __device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                      0);
    }
    static __device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                      0);
    }
};
// Eight elements of value 1 (the gain of a call without a gain tensor).
template <typename F> __device__ __forceinline__ u32x4 ones8() { return u32x4{F::kOnePair, F::kOnePair, F::kOnePair, F::kOnePair}; }

// Raw buffer descriptor over [p, p + bytes): accesses past the end read as zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, u32 bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// 16-byte load at byte offset `voff` (bounds-checked against the descriptor).
__device__ __forceinline__ u32x4 load16(__amdgpu_buffer_rsrc_t r, u32 voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
}

// Cache-policy operand of the buffer builtins on this target: bit 0 = sc0, bit 1 = nt, bit 4 = sc1.
constexpr int kCachePolicyNt = 2;
constexpr int kCachePolicySc1 = 16;

// The same for data that is read once per call (a streamed weight matrix): the non-temporal hint keeps it from
// displacing what the caches should hold (measured on the decode kernel: 3.5 % / 6 % faster on 32 / 235 MB of W).
__device__ __forceinline__ u32x4 load16_stream(__amdgpu_buffer_rsrc_t r, u32 voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, kCachePolicyNt);
}

// Device-coherent accesses for data handed from one workgroup to another inside a kernel.  On a
// multi-XCD part every XCD has its own L2: these accesses go through to the memory side instead
// of living in (or being served from) the issuing XCD's L2.
__device__ __forceinline__ void store_coherent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent2(float* p, float a, float b) {
    const f32x2 v = {a, b};
    __hip_atomic_store((unsigned long long*)p, __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x2 load_coherent2(const float* p) {
    const unsigned long long v =
        __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(f32x2, v);
}
// 16-byte versions, through a buffer descriptor over the exchanged array (the same for all lanes) and a byte
// offset per lane: the exchange of partial sums moves 16 bytes per lane and instruction instead of 8
// (measured on the decode kernel: 12.0 -> 11.4 us at 16 x 4096 x 4096, 9.5 -> 8.7 us at 16 x 1024 x 4096).
__device__ __forceinline__ void store_coherent4(__amdgpu_buffer_rsrc_t r, u32 byte_off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)byte_off, 0, kCachePolicySc1);
}
__device__ __forceinline__ f32x4 load_coherent4(__amdgpu_buffer_rsrc_t r, u32 byte_off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kCachePolicySc1));
}
// Blocks until every store this wavefront issued has been acknowledged by the memory system.
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float silu_f32(float a) {
    // a / (1 + exp(-a)); exp(-a) -> inf for very negative a gives a * 0 = -0.
    return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a));
}

}  // namespace prism
