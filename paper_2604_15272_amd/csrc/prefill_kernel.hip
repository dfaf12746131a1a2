// Prefill path: many rows of X, a compute-bound dense contraction on the bf16 matrix cores.
//
// A workgroup of four wavefronts (2 x 2) owns a BM x BN output tile and walks K in steps of 64.
// LDS holds two stages of a BM x 64 tile of X and a 64 x BN tile of W, both as
// [k / 8][row or column][8 k values], so that an MFMA operand is one 16-byte read and 32 consecutive
// lanes read 512 consecutive bytes.  On the way to LDS
//   - the raw squares of X are summed per row (the row reduction lives in the K-loop: paper
//     Figure 1(b), Accum beside Matmul);
//   - W, which arrives N-contiguous, is turned K-contiguous on 8 x 8 blocks held by one thread, and
//     the gain is folded in on the way: (X * g) W = X (g * W) row by row of W, so the multiply and
//     the re-rounding to bf16 ride on the transposition that W needs anyway (an element is
//     extracted, scaled by the gain of its row k and packed next to its K neighbour).  X then needs
//     no arithmetic besides its squares, which matters because only about four vector
//     instructions fit under one MFMA.
// The MFMA is issued "transposed" (W supplies the instruction's A operand, X its B operand), so a
// lane ends up with four consecutive output columns of one row, and its 1/rms factor (Table 1,
// "matmul commutes with div denominator") is one scalar per 32 x 32 block.
// The gated variant puts BN/2 columns of W1 and the same BN/2 columns of W2 side by side in the
// W tile; each wavefront holds matching W1 and W2 accumulators and applies SiLU(a) * b in registers.
//
// Software pipeline of one K step (four 16-deep MFMA phases), all in one wavefront's instruction
// stream because a 256 x 256 tile leaves one wavefront per SIMD:
//   phase 0..2: MFMAs of phase p run on operands read from LDS during phase p - 1, while the
//               operands of phase p + 1 are read, and a share of the NEXT tile is staged
//               (registers -> gain / squares / permutes -> the other LDS stage); each register set is
//               refilled from global memory with the tile after next as soon as it has been staged;
//   barrier;
//   phase 3:    MFMAs, while the first operands of the next tile are read from the other stage.
#include <type_traits>

#include "device_utils.h"
#include "prism_internal.h"

namespace prism {

namespace {

constexpr int BK = 64;       // K depth of one LDS stage
constexpr int KCH = BK / 8;  // 16-byte K chunks per row of a stage
constexpr int PAD = 1;       // slots of padding per chunk plane: eight planes then start 16 bytes apart mod 128,
                             // the spacing at which the eight-lanes-per-row X stores run at full LDS write rate

// Column swizzle of the W tile: a bijection on every aligned group of 16 columns (given the
// higher bits), chosen so that the permuted 8 x 8 blocks store without bank conflicts.
__device__ __forceinline__ int swz(int n) { return n ^ ((n >> 3) & 15); }

}  // namespace

template <int BM, int BN, bool GATED>
__global__ __launch_bounds__(256) void prefill_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ g,
                                                      const uint16_t* __restrict__ W1,
                                                      const uint16_t* __restrict__ W2, uint16_t* __restrict__ Y,
                                                      int M, int K, int N, float eps, int tiles_m, int tiles_n) {
    constexpr int WTM = BM / 2, WTN = BN / 2;        // wavefront tile
    constexpr int TM32 = WTM / 32, TN32 = WTN / 32;  // 32 x 32 MFMA blocks per wavefront
    constexpr int CW = GATED ? BN / 2 : BN;          // output columns per workgroup
    constexpr int XI = BM / 32;                      // 16-byte X loads per thread per stage
    constexpr int A_PLANE = BM + PAD, B_PLANE = BN + PAD;  // slots per chunk plane
    constexpr int A_SLOTS = KCH * A_PLANE, B_SLOTS = KCH * B_PLANE;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && BN <= 256, "tile shape");
    static_assert(!GATED || (WTN % 64 == 0), "gated tiles pair 32-column blocks of W1 and W2");
    static_assert(CW % 64 == 0, "a wavefront loads from one weight matrix only");

    extern __shared__ u32x4 lds[];
    u32x4* As = lds;                // [2][KCH][A_PLANE]
    u32x4* Bs = lds + 2 * A_SLOTS;  // [2][KCH][B_PLANE]
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
    // W: thread t owns one 8 (k) x 8 (n) block of the stage.  Which matrix a wavefront reads is the
    // same for all its lanes (CW is a multiple of 64); say so, to keep the descriptor in SGPRs.
    constexpr int NB8 = CW / 8;  // 8-column groups per weight matrix
    const int wmat = GATED ? __builtin_amdgcn_readfirstlane((tid / CW) & 1) : 0;
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
    // LDS slot of column j of the block, within a stage.  Threads without a block (tiles narrower than
    // 256) store to a padding slot instead of branching, which keeps the K loop one basic block.
    int w_dst[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w_dst[j] = w_active ? wkb * B_PLANE + swz(w_lds_col + j) : BN;

    u32x4 xreg[XI], wreg[8], g_cur, g_nxt;
    float ssq[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) ssq[i] = 0.f;

    // Global loads of K step kt (k past the end read as zero: X by predicate, g and W by the descriptor).
    auto load_g = [&](int kt) {  // gain of the eight rows (k values) of the thread's W block
        const int k = kt * BK + 8 * wkb;
        return load16(rg, (u32)k * 2u);  // past K is past the descriptor: zero
    };
    auto load_x = [&](int kt, int i) {
        const int k = kt * BK + 8 * xc;
        xreg[i] = load16(rx, (k < K) ? (u32)(((size_t)(xr0 + 32 * i) * K + k) * 2) : kOutOfRange);
    };
    auto load_w = [&](int kt) {
        const u32 woff = w_lane + (u32)kt * BK * row_bytes;
#pragma unroll
        for (int r = 0; r < 8; ++r) wreg[r] = load16(rw, woff + (u32)r * row_bytes);
    };

    auto load_w_row = [&](int kt, int r) {
        wreg[r] = load16(rw, w_lane + (u32)kt * BK * row_bytes + (u32)r * row_bytes);
    };

    // Staging of X chunk i, in four pieces (one dword = two elements each): the squares; the fourth
    // piece stores the 16 raw bytes to LDS.
    auto stage_x_piece = [&](u32x4* a_stage, int i, int d) {
        const u32 xx = xreg[i][d];
        ssq[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xx), __builtin_bit_cast(bf16x2, xx),
                                                 ssq[i], false);
        if (d == 3) a_stage[xc * A_PLANE + xr0 + 32 * i] = xreg[i];
    };
    // Staging of W column j of the thread's 8 x 8 block, in four pieces: piece t scales elements
    // (2t, j) and (2t + 1, j) by the gains of their rows and packs them as K neighbours (this is the
    // transposition); the fourth piece stores the 16 bytes to LDS.
    u32x4 wb;
    auto stage_w_piece = [&](u32x4* b_stage, int j, int t, const float (&gf)[8]) {
        const int d = j >> 1;
        const u32 w0 = wreg[2 * t][d], w1 = wreg[2 * t + 1][d];
        const float e0 = (j & 1) ? bf16_hi(w0) : bf16_lo(w0);
        const float e1 = (j & 1) ? bf16_hi(w1) : bf16_lo(w1);
        wb[t] = pack_bf16(e0 * gf[2 * t], e1 * gf[2 * t + 1]);
        if (t == 3) b_stage[w_dst[j]] = wb;
    };
    auto unpack_g = [&](u32x4 gg, float (&gf)[8]) {
#pragma unroll
        for (int d = 0; d < 4; ++d) { gf[2 * d] = bf16_lo(gg[d]); gf[2 * d + 1] = bf16_hi(gg[d]); }
    };

    // ---- LDS -> MFMA operand maps --------------------------------------------------------------
    int a_slot[TM32];  // X operand: row of the tile
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) a_slot[ib] = lh * A_PLANE + wm * WTM + 32 * ib + l32;
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
        b_slot[jb] = lh * B_PLANE + swz(col + l32);
    }
    // Operands of 16-deep phase kk of a stage: chunk plane 2 kk + lh.
    auto read_frags = [&](const u32x4* a_stage, const u32x4* b_stage, int kk, bf16x8 (&xf)[TM32], bf16x8 (&wf)[TN32]) {
#pragma unroll
        for (int ib = 0; ib < TM32; ++ib) xf[ib] = __builtin_bit_cast(bf16x8, a_stage[2 * kk * A_PLANE + a_slot[ib]]);
#pragma unroll
        for (int jb = 0; jb < TN32; ++jb) wf[jb] = __builtin_bit_cast(bf16x8, b_stage[2 * kk * B_PLANE + b_slot[jb]]);
    };

    f32x16 acc[TN32][TM32];
#pragma unroll
    for (int jb = 0; jb < TN32; ++jb)
#pragma unroll
        for (int ib = 0; ib < TM32; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][ib][v] = 0.f;
    constexpr int MF = TM32 * TN32;   // MFMAs per 16-deep phase
    constexpr int RD = TM32 + TN32;   // operand reads per phase
    constexpr int RPS = (RD + MF - 1) / MF;  // operand reads per MFMA slot (front-loaded)

    // One phase, as MF slots.  Slot q issues MFMA q on the operands read during the previous phase,
    // reads its share of the next operands (from `a_rd`/`b_rd`, 16-deep phase `kk_rd`), and does its
    // share of this phase's staging of the next tile: X pieces [XP0, XP0 + NXP) (piece = 4 * chunk +
    // dword; a finished chunk is refilled from the tile after next), W pieces [WP0, WP0 + NWP)
    // (piece = 4 * column + K pair), and, if TAIL, the refill of the W registers in the last slots.
    // A scheduling barrier closes every slot: the order written here is the order executed.
    auto phase = [&](auto xp0_c, auto nxp_c, auto wp0_c, auto nwp_c, auto tail_c, const u32x4* a_rd, const u32x4* b_rd,
                     int kk_rd, const bf16x8 (&xf)[TM32], const bf16x8 (&wf)[TN32], bf16x8 (&xf_n)[TM32],
                     bf16x8 (&wf_n)[TN32], u32x4* a_nxt, u32x4* b_nxt, const float (&gf)[8], int kt_load) {
        constexpr int XP0 = decltype(xp0_c)::value, NXP = decltype(nxp_c)::value, WP0 = decltype(wp0_c)::value,
                      NWP = decltype(nwp_c)::value, TAIL = decltype(tail_c)::value;
        constexpr int TAIL_SLOTS = TAIL ? (MF >= 8 ? 4 : 1) : 0;  // slots at the end that refill W rows
        constexpr int WS = MF - TAIL_SLOTS > 0 ? MF - TAIL_SLOTS : 1;  // slots that stage W pieces
#pragma unroll
        for (int q = 0; q < MF; ++q) {
            const int jb = q / TM32, ib = q % TM32;
            acc[jb][ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[jb], xf[ib], acc[jb][ib], 0, 0, 0);
#pragma unroll
            for (int r = q * RPS; r < (q + 1) * RPS && r < RD; ++r) {
                if (r < TM32) xf_n[r] = __builtin_bit_cast(bf16x8, a_rd[2 * kk_rd * A_PLANE + a_slot[r]]);
                else wf_n[r - TM32] = __builtin_bit_cast(bf16x8, b_rd[2 * kk_rd * B_PLANE + b_slot[r - TM32]]);
            }
#pragma unroll
            for (int it = (q * NXP) / MF; it < ((q + 1) * NXP) / MF; ++it) {
                const int i = (XP0 + it) / 4, d = (XP0 + it) % 4;
                stage_x_piece(a_nxt, i, d);
                if (d == 3) load_x(kt_load, i);
            }
            if (q < WS) {
#pragma unroll
                for (int it = (q * NWP) / WS; it < ((q + 1) * NWP) / WS; ++it)
                    stage_w_piece(b_nxt, (WP0 + it) / 4, (WP0 + it) % 4, gf);
            }
            if (TAIL && q >= MF - TAIL_SLOTS) {  // after the last W piece: refill the W rows
                constexpr int RPT = TAIL_SLOTS ? 8 / TAIL_SLOTS : 0;
#pragma unroll
                for (int r = (q - (MF - TAIL_SLOTS)) * RPT; r < (q - (MF - TAIL_SLOTS) + 1) * RPT; ++r)
                    load_w_row(kt_load, r);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::integral_constant;

    // X pieces (4 per chunk) and W pieces (4 per column) staged in phases 0, 1, 2.
    constexpr int xp0 = 0, xp1 = 2 * XI, xp2 = 3 * XI, xp3 = 4 * XI;
    constexpr int wp0 = 0, wp1 = 0, wp2 = 16, wp3 = 32;
    const int KT = (K + BK - 1) / BK;

    // ---- prologue: tile 0 to stage 0, tile 1 into registers, first operands ----------------------
    {
        g_cur = load_g(0);
#pragma unroll
        for (int i = 0; i < XI; ++i) load_x(0, i);
        load_w(0);
        float gf[8];
        unpack_g(g_cur, gf);
#pragma unroll
        for (int i = 0; i < XI; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d) stage_x_piece(As, i, d);
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t) stage_w_piece(Bs, j, t, gf);
        g_cur = load_g(1);
#pragma unroll
        for (int i = 0; i < XI; ++i) load_x(1, i);
        load_w(1);
    }
    __syncthreads();
    bf16x8 xfA[TM32], wfA[TN32], xfB[TM32], wfB[TN32];
    read_frags(As, Bs, 0, xfA, wfA);

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const u32x4* a_cur = As + cur * A_SLOTS;
        const u32x4* b_cur = Bs + cur * B_SLOTS;
        u32x4* a_nxt = As + (cur ^ 1) * A_SLOTS;
        u32x4* b_nxt = Bs + (cur ^ 1) * B_SLOTS;
        float gf[8];
        unpack_g(g_cur, gf);       // gain of tile kt + 1 (being staged)
        g_nxt = load_g(kt + 2);    // gain of the tile after next

        // Shares of the next tile per phase: X pieces [xp_p, xp_p+1), W pieces [wp_p, wp_p+1).  W starts
        // late: its registers are refilled last, so its loads have had the least time.
        phase(integral_constant<int, xp0>{}, integral_constant<int, xp1 - xp0>{}, integral_constant<int, wp0>{},
              integral_constant<int, wp1 - wp0>{}, integral_constant<int, 0>{}, a_cur, b_cur, 1, xfA, wfA, xfB, wfB,
              a_nxt, b_nxt, gf, kt + 2);
        phase(integral_constant<int, xp1>{}, integral_constant<int, xp2 - xp1>{}, integral_constant<int, wp1>{},
              integral_constant<int, wp2 - wp1>{}, integral_constant<int, 0>{}, a_cur, b_cur, 2, xfB, wfB, xfA, wfA,
              a_nxt, b_nxt, gf, kt + 2);
        phase(integral_constant<int, xp2>{}, integral_constant<int, xp3 - xp2>{}, integral_constant<int, wp2>{},
              integral_constant<int, wp3 - wp2>{}, integral_constant<int, 1>{}, a_cur, b_cur, 3, xfA, wfA, xfB, wfB,
              a_nxt, b_nxt, gf, kt + 2);
        __syncthreads();  // the next tile is complete in LDS; nobody reads the current stage any more
        phase(integral_constant<int, 0>{}, integral_constant<int, 0>{}, integral_constant<int, 0>{},
              integral_constant<int, 0>{}, integral_constant<int, 0>{}, a_nxt, b_nxt, 0, xfB, wfB, xfA, wfA, a_nxt,
              b_nxt, gf, kt + 2);
        g_cur = g_nxt;
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
