// Device-side helpers for gfx950: vector types, bf16 packing, buffer loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace prism {

typedef unsigned int u32;
typedef __attribute__((ext_vector_type(2))) u32 u32x2;
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

// Eight bf16 ones (the gain of a call without a gain tensor).
__device__ __forceinline__ u32x4 bf16_ones() { return u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u}; }

// Two floats -> two bf16 (round to nearest even) in one dword, a in the low half.
__device__ __forceinline__ u32 pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(u32, __builtin_convertvector(v, bf16x2));
}

// Raw buffer descriptor over [p, p + bytes): accesses past the end read as zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, u32 bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// 16-byte load at byte offset `voff` (bounds-checked against the descriptor).
__device__ __forceinline__ u32x4 load16(__amdgpu_buffer_rsrc_t r, u32 voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
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
// Blocks until every store this wavefront issued has been acknowledged by the memory system.
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float silu_f32(float a) {
    // a / (1 + exp(-a)); exp(-a) -> inf for very negative a gives a * 0 = -0.
    return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a));
}

}  // namespace prism
