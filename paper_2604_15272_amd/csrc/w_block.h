// A wavefront's 32 (k) x 128 (n) block of a row-major weight matrix, turned into MFMA B operands in
// registers.  Shared by the kernels that stream W once and keep few rows of the other operand
// (the decode kernel and the softmax kernel).
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

}  // namespace prism
