// A wavefront's 32 (k) x 128 (n) block of a row-major weight matrix, turned into MFMA B operands in
// registers, and the other pieces the kernels built on it share (the decode kernels, the softmax kernels,
// the attention kernel): they stream W once and keep few rows of the other operand.
#pragma once
#include "device_utils.h"

namespace prism {

// Lane (q, c), q = lane / 16, c = lane % 16, holds rows 8q .. 8q+7, columns 8c .. 8c+7 of the block.
struct WRows {
    u32x4 r[8];
};

// STREAM: the block is read by this workgroup only (non-temporal loads).
template <bool STREAM = false>
__device__ __forceinline__ void load_w_block(WRows& w, __amdgpu_buffer_rsrc_t rs, u32 voff, u32 row_bytes) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        w.r[i] = STREAM ? load16_stream(rs, voff + (u32)i * row_bytes) : load16(rs, voff + (u32)i * row_bytes);
}

// B operand j (j = 0..7) of a lane: column 8c + j of its 8 x 8 sub-block, eight K values.
template <int J>
__device__ __forceinline__ u32x4 b_operand(const WRows& w) {
    constexpr int d = J >> 1;
    constexpr u32 sel = (J & 1) ? 0x07060302u : 0x05040100u;
    u32x4 b;
    b[0] = __builtin_amdgcn_perm(w.r[1][d], w.r[0][d], sel);
    b[1] = __builtin_amdgcn_perm(w.r[3][d], w.r[2][d], sel);
    b[2] = __builtin_amdgcn_perm(w.r[5][d], w.r[4][d], sel);
    b[3] = __builtin_amdgcn_perm(w.r[7][d], w.r[6][d], sel);
    return b;
}

// A operand of a lane for a row of X scaled by the gain: x[8 K values] * g, rounded to the storage format;
// the raw squares are added to ss.
template <typename F>
__device__ __forceinline__ u32x4 scaled_a_operand(u32x4 x, u32x4 gg, float& ss) {
    u32x4 a;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const float x0 = F::lo(x[d]), x1 = F::hi(x[d]);
        ss = fmaf(x0, x0, ss);
        ss = fmaf(x1, x1, ss);
        a[d] = F::pack(x0 * F::lo(gg[d]), x1 * F::hi(gg[d]));
    }
    return a;
}

// The same operand in two parts, for calls whose error budget does not allow the rounding of x * g: the product of
// two stored values is exact in fp32 (8 + 8 or 11 + 11 significant bits), `hi` is that product rounded to the storage
// format and `lo` the rounded remainder, so hi + lo carries the product to 2^-17 (bf16) or 2^-23 (fp16) relative
// instead of 2^-9 / 2^-12, and (hi + lo) . W costs a second MFMA on the same B operand.  With a gain of exactly 1
// lo is zero.
template <typename F>
__device__ __forceinline__ void scaled_a_operand_split(u32x4 x, u32x4 gg, float& ss, u32x4& hi, u32x4& lo) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const float x0 = F::lo(x[d]), x1 = F::hi(x[d]);
        ss = fmaf(x0, x0, ss);
        ss = fmaf(x1, x1, ss);
        const float p0 = x0 * F::lo(gg[d]), p1 = x1 * F::hi(gg[d]);
        const u32 h = F::pack(p0, p1);
        hi[d] = h;
        // (a product beyond the format's range rounds to infinity: no remainder then, the result stays infinite)
        const float r0 = p0 - F::lo(h), r1 = p1 - F::hi(h);
        lo[d] = F::pack(__builtin_isfinite(r0) ? r0 : 0.f, __builtin_isfinite(r1) ? r1 : 0.f);
    }
}

// A wavefront's 16 x 128 accumulator tile (eight 16x16 MFMA results: accumulator j, element i of lane
// (q, c) is row 4q + i, column 8c + j) stored as rows of `pitch` floats at `tile`.  A lane owns 32 bytes
// of a row; lanes c and c + 8 are 256 bytes apart, the same banks: the upper eight write their second
// half first, so that one store instruction covers 16 different 16-byte bank groups.
__device__ __forceinline__ void store_acc_tile(float* tile, int pitch, int q, int c, const f32x4 (&acc)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float* dst = tile + (4 * q + i) * pitch + 8 * c;
        const f32x4 lo = f32x4{acc[0][i], acc[1][i], acc[2][i], acc[3][i]};
        const f32x4 hi = f32x4{acc[4][i], acc[5][i], acc[6][i], acc[7][i]};
        const bool upper = (c & 8) != 0;
        *(f32x4*)(dst + (upper ? 4 : 0)) = upper ? hi : lo;
        *(f32x4*)(dst + (upper ? 0 : 4)) = upper ? lo : hi;
    }
}

}  // namespace prism
