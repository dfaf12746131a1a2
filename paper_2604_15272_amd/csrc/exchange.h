// Partial results handed from one workgroup to another inside a kernel (split-K): CPT consecutive floats
// per lane, written through to the memory side and read from there (device-coherent accesses), in 16-byte
// pieces when CPT allows it.
#pragma once
#include "device_utils.h"

namespace prism {

// Descriptor over the exchanged array; byte offsets into it must stay below 2 GiB (the planner sees to it).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t exchange_rsrc(const float* base, size_t floats) {
    const size_t bytes = floats * 4;
    return make_rsrc(base, (u32)(bytes < 0x7FFFFFFFull ? bytes : 0x7FFFFFFFull));
}

template <int CPT>
__device__ __forceinline__ void store_partial(__amdgpu_buffer_rsrc_t r, float* base, size_t idx, const float (&v)[CPT]) {
    if constexpr (CPT % 4 == 0) {
#pragma unroll
        for (int e = 0; e < CPT; e += 4)
            store_coherent4(r, (u32)((idx + e) * 4), f32x4{v[e], v[e + 1], v[e + 2], v[e + 3]});
    } else {
#pragma unroll
        for (int e = 0; e < CPT; e += 2) store_coherent2(base + idx + e, v[e], v[e + 1]);
    }
}

template <int CPT>
__device__ __forceinline__ void load_partial(__amdgpu_buffer_rsrc_t r, const float* base, size_t idx, float (&v)[CPT]) {
    if constexpr (CPT % 4 == 0) {
#pragma unroll
        for (int e = 0; e < CPT; e += 4) {
            const f32x4 t = load_coherent4(r, (u32)((idx + e) * 4));
            v[e] = t[0];
            v[e + 1] = t[1];
            v[e + 2] = t[2];
            v[e + 3] = t[3];
        }
    } else {
#pragma unroll
        for (int e = 0; e < CPT; e += 2) {
            const f32x2 t = load_coherent2(base + idx + e);
            v[e] = t[0];
            v[e + 1] = t[1];
        }
    }
}

}  // namespace prism
