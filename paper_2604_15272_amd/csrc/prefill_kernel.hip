// Prefill path: many rows of X, a compute-bound dense contraction on the bf16 matrix cores.
//
// A workgroup of four wavefronts (2 x 2) owns a BM x BN output tile and walks K in steps of 64.
// Per step it stages a BM x 64 tile of X and a 64 x BN tile of W in LDS (double-buffered: the
// next step's global loads are issued before the current step's MFMAs and written to the other
// buffer after them).  On the way to LDS
//   - X is multiplied by the gain and re-rounded to bf16, and its raw squares are summed per row
//     (the row reduction lives in the K-loop: paper Figure 1(b), Accum beside Matmul);
//   - W, which arrives N-contiguous, is turned K-contiguous with byte permutes on 8 x 8 blocks.
// Both tiles sit in LDS as [k / 8][row or column][8 k values] so that an MFMA operand is one
// 16-byte read and 32 consecutive lanes read 512 consecutive bytes.
// The MFMA is issued "transposed" (W supplies the instruction's A operand, X its B operand), so a
// lane ends up with four consecutive output columns of one row, and its 1/rms factor (Table 1,
// "matmul commutes with div denominator") is one scalar per 32 x 32 block.
// The gated variant puts BN/2 columns of W1 and the same BN/2 columns of W2 side by side in the
// W tile; each wavefront holds matching W1 and W2 accumulators and applies SiLU(a) * b in registers.
#include "device_utils.h"
#include "prism_internal.h"

namespace prism {

namespace {

constexpr int BK = 64;       // K depth of one LDS stage
constexpr int KCH = BK / 8;  // 16-byte K chunks per row of a stage
constexpr int PAD = 2;       // slots of padding per chunk plane (spreads the X stores over banks)

// Column swizzle of the W tile: a bijection on every aligned group of 16 columns (given the
// higher bits), chosen so that the permuted 8 x 8 blocks store without bank conflicts.
__device__ __forceinline__ int swz(int n) { return n ^ ((n >> 3) & 15); }

}  // namespace

template <int BM, int BN, bool GATED>
__global__ __launch_bounds__(256) void prefill_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ g,
                                                      const uint16_t* __restrict__ W1,
                                                      const uint16_t* __restrict__ W2, uint16_t* __restrict__ Y,
                                                      int M, int K, int N, float eps, int tiles_m, int tiles_n) {
    constexpr int WTM = BM / 2, WTN = BN / 2;      // wavefront tile
    constexpr int TM32 = WTM / 32, TN32 = WTN / 32;  // 32 x 32 MFMA blocks per wavefront
    constexpr int CW = GATED ? BN / 2 : BN;        // output columns per workgroup
    constexpr int XI = BM / 32;                    // 16-byte X loads per thread per stage
    constexpr int A_PLANE = BM + PAD, B_PLANE = BN + PAD;  // slots per chunk plane
    constexpr int A_SLOTS = KCH * A_PLANE, B_SLOTS = KCH * B_PLANE;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && BN <= 256, "tile shape");
    static_assert(!GATED || (WTN % 64 == 0), "gated tiles pair 32-column blocks of W1 and W2");
    static_assert(CW % 64 == 0, "a wavefront loads from one weight matrix only");

    extern __shared__ u32x4 lds[];
    u32x4* As = lds;                 // [2][KCH][A_PLANE]
    u32x4* Bs = lds + 2 * A_SLOTS;   // [2][KCH][B_PLANE]
    float* rscale = (float*)(lds + 2 * A_SLOTS + 2 * B_SLOTS);  // [BM]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    // Tile order: consecutive workgroups share a column tile of W and walk down the rows.
    const int tile = blockIdx.x;
    const int tm = tile % tiles_m, tn = tile / tiles_m;
    const int m0 = tm * BM, n0 = tn * CW;

    // ---- global -> register staging maps -------------------------------------------------------
    // X: thread t loads row (t / 8 + 32 i), K chunk (t % 8) of the stage.
    const int xr0 = tid >> 3, xc = tid & 7;
    const size_t x_first = (size_t)m0 * K;
    const size_t x_left = ((size_t)M * K - x_first) * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + x_first, (u32)(x_left < 0x7FFFFFFFull ? x_left : 0x7FFFFFFFull));
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(g, (u32)K * 2u);
    // W: thread t owns one 8 (k) x 8 (n) block of the stage.
    constexpr int NB8 = CW / 8;  // 8-column groups per weight matrix
    const int wmat = GATED ? (tid / CW) & 1 : 0;  // wavefront-uniform: CW is a multiple of 64
    const int wt = GATED ? tid % CW : tid;
    const bool w_active = tid < BN;
    const int wkb = wt / NB8, wnb = wt % NB8;
    const bool w_col_ok = w_active && (n0 + 8 * wnb) < N;
    const size_t w_left = ((size_t)K * N - n0) * 2;
    const u32 w_bytes = (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc((wmat ? W2 : W1) + n0, w_bytes);
    const u32 row_bytes = (u32)N * 2u;
    const u32 w_lane = w_col_ok ? ((u32)(8 * wkb) * row_bytes + (u32)(16 * wnb)) : kOutOfRange;
    const int w_lds_col = wmat * (BN / 2) + 8 * wnb;  // first LDS column of the block

    u32x4 xreg[XI], greg;
    u32x4 wreg[8];
    float ssq[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) ssq[i] = 0.f;

    auto issue_loads = [&](int kt) {
        const int k = kt * BK + 8 * xc;
        const bool k_ok = k < K;
        greg = load16(rg, k_ok ? (u32)k * 2u : kOutOfRange);
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            const int r = xr0 + 32 * i;
            xreg[i] = load16(rx, k_ok ? (u32)(((size_t)r * K + k) * 2) : kOutOfRange);
        }
        const u32 woff = w_lane + (u32)kt * BK * row_bytes;
#pragma unroll
        for (int r = 0; r < 8; ++r) wreg[r] = load16(rw, woff + (u32)r * row_bytes);
    };

    auto stage_to_lds = [&](int buf) {
        u32x4* a_dst = As + buf * A_SLOTS + xc * A_PLANE;
        float gf[8];
#pragma unroll
        for (int d = 0; d < 4; ++d) { gf[2 * d] = bf16_lo(greg[d]); gf[2 * d + 1] = bf16_hi(greg[d]); }
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            u32x4 a;
            float s = ssq[i];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float x0 = bf16_lo(xreg[i][d]), x1 = bf16_hi(xreg[i][d]);
                s = fmaf(x0, x0, s);
                s = fmaf(x1, x1, s);
                a[d] = pack_bf16(x0 * gf[2 * d], x1 * gf[2 * d + 1]);
            }
            ssq[i] = s;
            a_dst[xr0 + 32 * i] = a;
        }
        if (w_active) {
            u32x4* b_dst = Bs + buf * B_SLOTS + wkb * B_PLANE;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int d = j >> 1;
                const u32 sel = (j & 1) ? 0x07060302u : 0x05040100u;
                u32x4 b;
                b[0] = __builtin_amdgcn_perm(wreg[1][d], wreg[0][d], sel);
                b[1] = __builtin_amdgcn_perm(wreg[3][d], wreg[2][d], sel);
                b[2] = __builtin_amdgcn_perm(wreg[5][d], wreg[4][d], sel);
                b[3] = __builtin_amdgcn_perm(wreg[7][d], wreg[6][d], sel);
                b_dst[swz(w_lds_col + j)] = b;
            }
        }
    };

    // ---- LDS -> MFMA operand maps --------------------------------------------------------------
    int a_slot[TM32];  // X operand: row of the tile
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) a_slot[ib] = wm * WTM + 32 * ib + l32;
    int b_slot[TN32];  // W operand: swizzled column of the tile
#pragma unroll
    for (int jb = 0; jb < TN32; ++jb) {
        int col;
        if (GATED) {
            constexpr int H = TN32 / 2;
            col = (jb < H) ? (wn * (WTN / 2) + 32 * jb) : (BN / 2 + wn * (WTN / 2) + 32 * (jb - H));
        } else {
            col = wn * WTN + 32 * jb;
        }
        b_slot[jb] = swz(col + l32);
    }

    f32x16 acc[TN32][TM32];
#pragma unroll
    for (int jb = 0; jb < TN32; ++jb)
#pragma unroll
        for (int ib = 0; ib < TM32; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][ib][v] = 0.f;

    const int KT = (K + BK - 1) / BK;
    issue_loads(0);
    stage_to_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        const bool more = (kt + 1) < KT;
        if (more) issue_loads(kt + 1);

        const u32x4* a_src = As + buf * A_SLOTS;
        const u32x4* b_src = Bs + buf * B_SLOTS;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int ch = 2 * kk + lh;
            bf16x8 xf[TM32], wf[TN32];
#pragma unroll
            for (int ib = 0; ib < TM32; ++ib) xf[ib] = __builtin_bit_cast(bf16x8, a_src[ch * A_PLANE + a_slot[ib]]);
#pragma unroll
            for (int jb = 0; jb < TN32; ++jb) wf[jb] = __builtin_bit_cast(bf16x8, b_src[ch * B_PLANE + b_slot[jb]]);
#pragma unroll
            for (int jb = 0; jb < TN32; ++jb)
#pragma unroll
                for (int ib = 0; ib < TM32; ++ib)
                    acc[jb][ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[jb], xf[ib], acc[jb][ib], 0, 0, 0);
        }

        if (more) stage_to_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- 1/rms per row: the eight threads that shared a row combine their partial sums -----------
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        float s = ssq[i];
        s += __shfl_xor(s, 1, 64);
        s += __shfl_xor(s, 2, 64);
        s += __shfl_xor(s, 4, 64);
        if (xc == 0) rscale[xr0 + 32 * i] = __builtin_amdgcn_rsqf(s / (float)K + eps);
    }
    __syncthreads();

    // ---- epilogue: register v of block (jb, ib) is row 32 ib + l32, column 32 jb + 8 (v / 4) + 4 lh + v % 4
    constexpr int OB = GATED ? TN32 / 2 : TN32;  // output 32-column blocks per wavefront
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) {
        const int ml = wm * WTM + 32 * ib + l32;
        const int m = m0 + ml;
        const float r = rscale[ml];
        if (m >= M) continue;
#pragma unroll
        for (int jb = 0; jb < OB; ++jb) {
            const int cbase = n0 + wn * (GATED ? WTN / 2 : WTN) + 32 * jb + 4 * lh;
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int n = cbase + 8 * vg;
                if (n >= N) continue;
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    y[e] = acc[jb][ib][4 * vg + e] * r;
                    if (GATED) y[e] = silu_f32(y[e]) * (acc[jb + OB][ib][4 * vg + e] * r);
                }
                *(u32x2*)(Y + (size_t)m * N + n) = u32x2{pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
            }
        }
    }
}

template <int BM, int BN, bool GATED>
static hipError_t launch_tile(const Call& c) {
    constexpr int CW = GATED ? BN / 2 : BN;
    const int tiles_m = (c.M + BM - 1) / BM, tiles_n = (c.N + CW - 1) / CW;
    const size_t lds = (size_t)(2 * KCH * (BM + PAD) + 2 * KCH * (BN + PAD)) * 16 + (size_t)BM * 4;
    auto kern = prefill_kernel<BM, BN, GATED>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), lds, c.stream, (const uint16_t*)c.X,
                       (const uint16_t*)c.g, (const uint16_t*)c.W1, (const uint16_t*)(c.gated ? c.W2 : c.W1),
                       (uint16_t*)c.Y, c.M, c.K, c.N, c.eps, tiles_m, tiles_n);
    return hipGetLastError();
}

hipError_t launch_prefill_bf16(const Call& c, int tile_m, int tile_n) {
    if (c.gated) {
        if (tile_m == 256 && tile_n == 256) return launch_tile<256, 256, true>(c);
        if (tile_m == 128 && tile_n == 256) return launch_tile<128, 256, true>(c);
        if (tile_m == 128 && tile_n == 128) return launch_tile<128, 128, true>(c);
    } else {
        if (tile_m == 256 && tile_n == 256) return launch_tile<256, 256, false>(c);
        if (tile_m == 256 && tile_n == 192) return launch_tile<256, 192, false>(c);
        if (tile_m == 128 && tile_n == 128) return launch_tile<128, 128, false>(c);
        if (tile_m == 64 && tile_n == 64) return launch_tile<64, 64, false>(c);
    }
    return hipErrorInvalidValue;
}

}  // namespace prism
