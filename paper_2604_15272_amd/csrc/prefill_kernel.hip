// Prefill path: many rows of X, a compute-bound dense contraction on the bf16 matrix cores.
//
// A workgroup of four wavefronts (2 x 2) owns a BM x BN output tile and walks K in steps of 64.
// LDS holds two stages of a BM x 64 tile of X and a 64 x BN tile of W; an MFMA operand (8 K values of
// one row or column) is one 16-byte read.
//   - X goes from global memory straight into LDS (buffer loads with the LDS flag: no registers, no
//     vector instructions, no LDS store instructions).  Such a load writes the 64 lanes' 16 bytes
//     back to back, so a stage is row-major (8 rows = 1 KiB per wavefront instruction); to keep the
//     operand reads (32 consecutive rows, same K chunk) off each other's banks, the K chunks of row r
//     are rotated by r % 8 (done on the global address, which is free) and every group of 8 rows
//     is followed by 128 bytes of padding.
//   - W sits in LDS as [k / 8][column][8 k values].
//   - W, which arrives N-contiguous, is turned K-contiguous on 8 x 8 blocks held by one thread, and
//     the gain is folded in on the way: (X * g) W = X (g * W) row by row of W, so the multiply and
//     the re-rounding to bf16 ride on the transposition that W needs anyway (an element is
//     extracted, scaled by the gain of its row k and packed next to its K neighbour).  X then needs
//     no vector arithmetic at all, which matters because only about four vector instructions fit
//     under one MFMA.
// The row sums of squares live in the K-loop too (paper Figure 1(b), Accum beside Matmul), but on the
// matrix cores: a 4x4x4 MFMA fed the same X operand registers on both sides yields, on its diagonal,
// the squares of four K values per lane, and accumulates them.  (A dot-product instruction would be
// one vector op per two elements, but measured here it cannot overlap with a running MFMA and cost
// 13 % of the kernel; two small MFMAs per operand cost 16 cycles of the matrix pipe.)  The two
// wavefronts that share rows take alternate 16-deep phases.
// The MFMA is issued "transposed" (W supplies the instruction's A operand, X its B operand), so a
// lane ends up with four consecutive output columns of one row, and its 1/rms factor (Table 1,
// "matmul commutes with div denominator") is one scalar per 32 x 32 block.
// The gated variant puts BN/2 columns of W1 and the same BN/2 columns of W2 side by side in the
// W tile; each wavefront holds matching W1 and W2 accumulators and applies SiLU(a) * b in registers.
//
// Software pipeline of one K step (four 16-deep MFMA phases of MF MFMAs each), all in one wavefront's
// instruction stream because a 256 x 256 tile leaves one wavefront per SIMD.  Every MFMA is a "slot"
// closed by a scheduling barrier, and the other work is dealt out to the slots:
//   - operands: the MFMAs of a phase run on registers read from LDS during the phase before;
//   - W staging: two register sets alternate.  While the tile in one set is scaled, transposed and
//     stored to the other LDS stage (phases 0..2, a few vector instructions per slot), the other set
//     is being loaded with the tile after it;
//   - global memory: the X requests of the tile after next and the loads of the W set just staged are
//     spread over phase 3 and phases 0, 1 of the following step (requests first), one instruction
//     every few slots; the four wavefronts run the same schedule, and bunched loads would block the
//     MFMAs behind them at the address unit;
//   - barrier after phase 2: written as explicit waits plus s_barrier.  It waits for this wavefront's
//     LDS accesses and for its X requests of the next tile (all but the loads issued after them;
//     loads complete in issue order), not for loads that are needed later.
// The prologue issues its global-memory instructions in the same order as the loop, so that the
// wait counts the compiler derives for the loop body are the steady-state ones.
// Measured on MI355X (4096 x 4096 x 2*14336 gated): the shader clock drops from 2.3 GHz to 1.55 - 1.75
// GHz when all 256 CUs run this kernel, and a K step takes about 3070 cycles against 2176 of pure
// MFMA work; the vendor GEMM library reaches 1.27 PFLOP/s on the same plain product in this layout.
#include <type_traits>

#include "device_utils.h"
#include "prism_internal.h"


namespace prism {

namespace {

// One row of a thread's block of W: 8 columns (16 bytes) or 6 (12 bytes; the fourth dword is unused).
template <int CB> __device__ __forceinline__ u32x4 load_cols(__amdgpu_buffer_rsrc_t r, u32 voff) {
    if constexpr (CB == 8) {
        return load16(r, voff);
    } else {
        const u32x3 v = __builtin_amdgcn_raw_buffer_load_b96(r, (int)voff, 0, 0);
        return u32x4{v[0], v[1], v[2], 0u};
    }
}

constexpr int BK = 64;       // K depth of one LDS stage
constexpr int KCH = BK / 8;  // 16-byte K chunks per row of a stage
constexpr int PAD = 1;       // 16-byte slots of padding per K-chunk plane of the W stage
constexpr int XGS = 72;      // 16-byte slots per group of 8 rows of the X stage: 64 of data, 8 of padding

// Column swizzle of the W tile: a bijection on every aligned group of 16 columns (given the
// higher bits), so that operand reads of consecutive columns stay conflict-free, chosen so that
// the stores of the transposed blocks are conflict-free too.  With 8-column blocks sixteen lanes
// store columns 8 i + j: an XOR with the group number separates them.  With 6-column blocks
// (192-wide tile) they store columns 6 i + j, whose positions within a group of 16 repeat after
// 48 columns: every other run of three groups is rotated by one.
template <int CB> __device__ __forceinline__ int swz(int n) {
    if constexpr (CB == 8) return n ^ ((n >> 3) & 15);
    else return (n & ~15) | ((n + (((n >> 4) / 3) & 1)) & 15);
}

}  // namespace

template <typename F, int BM, int BN, bool GATED>
__global__ __launch_bounds__(256) void prefill_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ g,
                                                      const uint16_t* __restrict__ W1,
                                                      const uint16_t* __restrict__ W2, uint16_t* __restrict__ Y,
                                                      int M, int K, int N, float eps, int tiles_m, int tiles_n, int flags) {
    constexpr int WTM = BM / 2, WTN = BN / 2;        // wavefront tile
    constexpr int TM32 = WTM / 32, TN32 = WTN / 32;  // 32 x 32 MFMA blocks per wavefront
    constexpr int CW = GATED ? BN / 2 : BN;          // output columns per workgroup
    constexpr int XI = BM / 32;                      // 16-byte X loads per thread per stage
    constexpr int B_PLANE = BN + PAD;                      // slots per chunk plane of W
    constexpr int A_SLOTS = (BM / 8) * XGS, B_SLOTS = KCH * B_PLANE;  // slots per stage
    static_assert(BM % 64 == 0 && BN % 64 == 0 && BN <= 256, "tile shape");
    static_assert(!GATED || (WTN % 64 == 0), "gated tiles pair 32-column blocks of W1 and W2");
    static_assert(CW % 64 == 0, "a wavefront loads from one weight matrix only");

    extern __shared__ u32x4 lds[];
    u32x4* As = lds;                // [2][BM / 8][XGS]
    u32x4* Bs = lds + 2 * A_SLOTS;  // [2][KCH][B_PLANE]
    float* rscale = (float*)(lds + 2 * A_SLOTS + 2 * B_SLOTS);  // [BM]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin and each XCD has its own L2, so
    // the 32 workgroups that run together on one XCD should share as much of X and W as they can: a
    // block of 4 row tiles x 8 column tiles needs 12 tile streams instead of the 18 or more of a strip.
    //   1. position: within each full round of 256 workgroups, XCD x (ids = x mod 8) takes the 32
    //      consecutive positions 32 x .. 32 x + 31 (a partial last round is split into 8 equal runs,
    //      its remainder keeps the identity);
    //   2. tile: positions fill bands of 8 column tiles row by row, so 32 consecutive positions are
    //      such a 4 x 8 block.
    int pos = blockIdx.x;
    {
        const int total = tiles_m * tiles_n, full = total & ~255;
        if (pos < full) {
            pos = (pos & ~255) + (pos & 7) * 32 + ((pos & 255) >> 3);
        } else {
            const int run = (total - full) >> 3, b = pos - full;
            if (b < 8 * run) pos = full + (b & 7) * run + (b >> 3);
        }
    }
    const int band = pos / (8 * tiles_m), in_band = pos % (8 * tiles_m);
    const int band_w = tiles_n - 8 * band < 8 ? tiles_n - 8 * band : 8;
    const int tm = in_band / band_w, tn = 8 * band + in_band % band_w;
    const int m0 = tm * BM, n0 = tn * CW;

    // ---- global -> register staging maps -------------------------------------------------------
    // X: thread t requests row (t / 8 + 32 i) of the stage.
    const int xr0 = tid >> 3;
    const size_t x_first = (size_t)m0 * K;
    const size_t x_left = ((size_t)M * K - x_first) * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(X + x_first, (u32)(x_left < 0x7FFFFFFFull ? x_left : 0x7FFFFFFFull));
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(g, (u32)K * 2u);
    // W: thread t owns one 8 (k) x CB (n) block of the stage, CB = 8 columns (one 16-byte load per
    // row).  A 192-column tile would leave a quarter of the threads without a block while the others
    // carry the whole transposition, which is more vector work than fits under their 48 MFMAs per K
    // step; there a block is 6 columns wide (12-byte loads), so that all 256 threads share the work.
    // Which matrix a wavefront reads is the same for all its lanes (a matrix's threads are a multiple of 64);
    // say so, to keep the descriptor in SGPRs.
    // A 128-column tile (or 2 x 64 gated) has only 128 such blocks: two of the four wavefronts would carry the
    // whole transposition (160 vector instructions per K step beside 16 MFMAs) and the step would take as long
    // as they do.  There a block is 4 (k) x 8 (n): two threads share a column's 16-byte operand, each storing
    // its 8-byte half.
    constexpr int CB = (BN == 192) ? 6 : 8;
    constexpr int NBG = CW / CB;     // column groups per weight matrix
    constexpr int KR = ((GATED ? 2 : 1) * KCH * NBG <= 128) ? 4 : 8;  // k rows of a thread's block
    constexpr int KQ = BK / KR;      // blocks per column group along k
    constexpr int TPM = KQ * NBG;    // threads per weight matrix
    constexpr int NP = (KR / 2) * CB;  // staging pieces per thread and tile (one per pair of k rows and column)
    static_assert(CW % CB == 0 && TPM % 64 == 0 && (GATED ? 2 : 1) * TPM <= 256, "W staging map");
    const int wmat = GATED ? __builtin_amdgcn_readfirstlane((tid / TPM) & 1) : 0;
    const int wt = GATED ? tid % TPM : tid;
    const bool w_active = tid < (GATED ? 2 : 1) * TPM;
    const int wkq = wt / NBG, wnb = wt % NBG;          // the thread's block: k rows KR wkq .. KR wkq + KR - 1
    const int wkb = wkq / (8 / KR), whalf = wkq % (8 / KR);  // the 8-deep chunk plane it belongs to, and which half
    // (A 6-column group that straddles N reads columns that belong to the next row of W: they only
    // reach accumulators of columns >= N, which are never stored.)
    const bool w_col_ok = w_active && (n0 + CB * wnb) < N;
    const size_t w_left = ((size_t)K * N - n0) * 2;
    const u32 w_bytes = (u32)(w_left < 0x7FFFFFFFull ? w_left : 0x7FFFFFFFull);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc((wmat ? W2 : W1) + n0, w_bytes);
    const u32 row_bytes = (u32)N * 2u;
    const u32 w_lane = w_col_ok ? ((u32)(KR * wkq) * row_bytes + (u32)(2 * CB * wnb)) : kOutOfRange;
    const int w_lds_col = wmat * (BN / 2) + CB * wnb;  // first LDS column of the block
    // LDS slot of column j of the block, within a stage.  Threads without a block (tiles narrower than
    // 256) store to a padding slot instead of branching, which keeps the K loop one basic block.
    int w_dst[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) w_dst[j] = w_active ? wkb * B_PLANE + swz<CB>(w_lds_col + j) : BN;

    // Two register sets for W: while one is being staged into LDS, the other already holds the tile
    // after it, so a tile's loads have more than a whole K step to arrive.
    struct WSet {
        u32x4 w[KR];  // the rows of the thread's block of W
        u32x4 g;      // gain of those rows (the first KR / 2 dwords)
    };
    WSet ws_a, ws_b;
    const bool has_gain = (flags & kFlagGain) != 0;

    // Global loads of K step kt (k past the end read as zero: X by predicate, g and W by the descriptor).
    // Load 0 of a set is the gain, loads 1..8 are the rows.
    auto load_w = [&](WSet& s, int kt, int i) {
        if (i == 0) {
            // Without a gain tensor the load is still issued (out of range: it returns zero and touches
            // no memory): the wait counts of the pipeline below count instructions.
            const u32 goff = has_gain ? (u32)(kt * BK + KR * wkq) * 2u : kOutOfRange;
            u32x4 v;
            if constexpr (KR == 8) {
                v = load16(rg, goff);
            } else {
                const u32x2 h = __builtin_amdgcn_raw_buffer_load_b64(rg, (int)goff, 0, 0);
                v = u32x4{h[0], h[1], 0u, 0u};
            }
            const u32x4 one = ones8<F>();
            s.g = u32x4{has_gain ? v[0] : one[0], has_gain ? v[1] : one[1], has_gain ? v[2] : one[2],
                        has_gain ? v[3] : one[3]};
        }
        else s.w[i - 1] = load_cols<CB>(rw, w_lane + (u32)kt * BK * row_bytes + (u32)(i - 1) * row_bytes);
    };
    constexpr int NWL = KR + 1;  // loads per set
    // X, request i of K step kt: this wavefront moves rows 8 * wave + 32 i .. + 7 (64 K values each)
    // into group wave + 4 i of the stage; lane l = 8 r + p fetches chunk p ^ r of its row.
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int x_chunk = (lane & 7) ^ (lane >> 3);
    auto request_x = [&](u32x4* a_stage, int kt, int i) {
        const int k = kt * BK + 8 * x_chunk;
        const u32 voff = (k < K) ? (u32)(((size_t)(xr0 + 32 * i) * K + k) * 2) : kOutOfRange;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(a_stage + (wave_s + 4 * i) * XGS),
                                                 16, (int)voff, 0, 0, 0);
    };

    // Staging of W column j of the thread's 8 x 8 block, in four pieces: piece t scales elements
    // (2t, j) and (2t + 1, j) by the gains of their rows and packs them as K neighbours (this is the
    // transposition); the fourth piece stores the 16 bytes to LDS.
    u32x4 wb;
    auto stage_w_piece = [&](const WSet& s, u32x4* b_stage, int j, int t) {
        const int d = j >> 1;
        const u32 w0 = s.w[2 * t][d], w1 = s.w[2 * t + 1][d], gg = s.g[t];
        const float e0 = (j & 1) ? F::hi(w0) : F::lo(w0);
        const float e1 = (j & 1) ? F::hi(w1) : F::lo(w1);
        wb[t] = F::pack(e0 * F::lo(gg), e1 * F::hi(gg));
        if constexpr (KR == 8) {
            if (t == 3) b_stage[w_dst[j]] = wb;
        } else {
            if (t == 1) ((u32x2*)(b_stage + w_dst[j]))[whalf] = u32x2{wb[0], wb[1]};
        }
    };

    // ---- LDS -> MFMA operand maps --------------------------------------------------------------
    // X operand of 32-row block ib in 16-deep phase kk: row R = wm * WTM + 32 ib + l32, chunk 2 kk + lh,
    // which sits at position (2 kk + lh) ^ (R % 8) of its row: slot a_slot[kk] + 4 * XGS * ib.
    int a_slot[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk)
        a_slot[kk] = (wm * (WTM / 8) + (l32 >> 3)) * XGS + (l32 & 7) * 8 + ((2 * kk + lh) ^ (l32 & 7));
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
        b_slot[jb] = lh * B_PLANE + swz<CB>(col + l32);
    }
    // Operands of 16-deep phase kk of a stage: chunk plane 2 kk + lh.
    auto read_frags = [&](const u32x4* a_stage, const u32x4* b_stage, int kk, u32x4 (&xf)[TM32], u32x4 (&wf)[TN32]) {
#pragma unroll
        for (int ib = 0; ib < TM32; ++ib) xf[ib] = a_stage[a_slot[kk] + 4 * XGS * ib];
#pragma unroll
        for (int jb = 0; jb < TN32; ++jb) wf[jb] = b_stage[2 * kk * B_PLANE + b_slot[jb]];
    };

    f32x16 acc[TN32][TM32];
#pragma unroll
    for (int jb = 0; jb < TN32; ++jb)
#pragma unroll
        for (int ib = 0; ib < TM32; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jb][ib][v] = 0.f;
    // Sums of squares: gram[ib][lane % 4] accumulates the squares of the K values this lane's operand
    // registers have held for row 32 ib + lane % 32 (in the phases this wavefront is in charge of).
    f32x4 gram[TM32];
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) gram[ib] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int wn_s = __builtin_amdgcn_readfirstlane(wn);

    constexpr int MF = TM32 * TN32;          // MFMAs per 16-deep phase
    constexpr int RD = TM32 + TN32;          // operand reads per phase
    constexpr int RPS = (RD + MF - 1) / MF;  // operand reads per MFMA slot (front-loaded)

    // Global-memory instructions that bring in one more tile ("refill"): the XI requests of an X tile,
    // then the NWL loads of the W set one tile later - NI instructions, spread evenly
    // over the 3 MF slots of three consecutive phases (phase 3 of one K step, phases 0 and 1 of the
    // next).  All four wavefronts run this schedule at the same time and the address unit takes about
    // 16 cycles per instruction, so bunching them would block the MFMAs queued behind them.
    // The requests come first: the barrier that needs them then leaves the NWL loads after them in
    // flight.
    constexpr int NI = XI + NWL;
    auto refill_slot = [&](auto part_c, int q, u32x4* a_x, int kt_x, WSet& w_ld) {
        constexpr int PART = decltype(part_c)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if ((i * 3 * MF) / NI != PART * MF + q) continue;
            if (i < XI) request_x(a_x, kt_x, i);
            else load_w(w_ld, kt_x + 1, i - XI);
            // A small tile puts several of these instructions into one slot; the wait counts below depend on
            // their order (requests before loads), so nothing may be moved across any of them.
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One phase, as MF slots.  Slot q issues MFMA q on the operands read during the previous phase,
    // reads its share of the next operands (from `a_rd`/`b_rd`, 16-deep phase `kk_rd`), and does its
    // share of this phase's work on the tiles to come: part PART of the refill (none if negative) of
    // X tile `kt_x` into stage `a_x` and of W tile `kt_x` + 1 into the set `w_ld`; W pieces
    // [WP0, WP0 + NWP) (piece = (KR / 2) * column + K pair) of the set `w_st` staged into `b_st`.  A
    // scheduling barrier closes every slot: the order written here is the order executed.
    auto phase = [&](auto kk_c, auto part_c, auto wp0_c, auto nwp_c, const u32x4* a_rd, const u32x4* b_rd,
                     int kk_rd, const u32x4 (&xf)[TM32], const u32x4 (&wf)[TN32], u32x4 (&xf_n)[TM32],
                     u32x4 (&wf_n)[TN32], u32x4* a_x, int kt_x, WSet& w_ld, const WSet& w_st, u32x4* b_st) {
        constexpr int KK = decltype(kk_c)::value, PART = decltype(part_c)::value, WP0 = decltype(wp0_c)::value,
                      NWP = decltype(nwp_c)::value;
        // Sums of squares on the matrix cores, in the phases this wavefront is in charge of.  Written
        // as assembly so that these accumulators stay in ordinary vector registers: the 256
        // accumulators of the product fill the accumulation registers, and the compiler would shuttle
        // them out and back to make room.  The trailing wait states cover a dependent MFMA that
        // follows at once (same accumulator, next K half) when a wavefront has few row blocks.
        if (wn_s == (KK & 1)) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int ib = 0; ib < TM32; ++ib) {
                    const u32x2 v = {xf[ib][2 * h], xf[ib][2 * h + 1]};
                    constexpr bool kBf16 = std::is_same<F, Bf16>::value;
                    if constexpr (TM32 >= 4) {  // three other MFMAs separate the two uses of an accumulator
                        if constexpr (kBf16) asm volatile("v_mfma_f32_4x4x4_16b_bf16 %0, %1, %1, %0" : "+v"(gram[ib]) : "v"(v));
                        else asm volatile("v_mfma_f32_4x4x4_16b_f16 %0, %1, %1, %0" : "+v"(gram[ib]) : "v"(v));
                    } else {
                        if constexpr (kBf16)
                            asm volatile("v_mfma_f32_4x4x4_16b_bf16 %0, %1, %1, %0\n\ts_nop 4" : "+v"(gram[ib]) : "v"(v));
                        else
                            asm volatile("v_mfma_f32_4x4x4_16b_f16 %0, %1, %1, %0\n\ts_nop 4" : "+v"(gram[ib]) : "v"(v));
                    }
                }
        }
#pragma unroll
        for (int q = 0; q < MF; ++q) {
            const int jb = q / TM32, ib = q % TM32;
            acc[jb][ib] = F::mfma_32x32x16(wf[jb], xf[ib], acc[jb][ib]);
#pragma unroll
            for (int r = q * RPS; r < (q + 1) * RPS && r < RD; ++r) {
                if (r < TM32) xf_n[r] = a_rd[a_slot[kk_rd] + 4 * XGS * r];
                else wf_n[r - TM32] = b_rd[2 * kk_rd * B_PLANE + b_slot[r - TM32]];
            }
            if constexpr (PART >= 0) refill_slot(part_c, q, a_x, kt_x, w_ld);
#pragma unroll
            for (int it = (q * NWP) / MF; it < ((q + 1) * NWP) / MF; ++it)
                stage_w_piece(w_st, b_st, (WP0 + it) / (KR / 2), (WP0 + it) % (KR / 2));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::integral_constant;
    // Barrier between K steps.  Written out instead of __syncthreads(): the fences of the latter make
    // the compiler wait for every LDS-writing load in flight, also those of a tile that is not needed
    // yet.  What the barrier has to order is stated here instead: this wavefront's LDS writes and reads are complete (lgkmcnt), and so are its X
    // requests of the next tile - everything but the newest `younger` global-memory instructions; they
    // complete in issue order.
    auto stage_barrier = [&](auto younger_c) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(decltype(younger_c)::value) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // W pieces (KR / 2 per column, NP per tile): the first P3 could be staged a step early, in phase 3 (after
    // the barrier, into the stage just vacated), the rest in phases 0, 1, 2.  Measured best with none
    // in phase 3: the set's last loads are issued only two phases before it.
    constexpr int P3 = 0;
    constexpr int wp1 = P3 + (NP - P3) / 3, wp2 = P3 + 2 * (NP - P3) / 3;
    const int KT = (K + BK - 1) / BK;
    const int KT2 = (KT + 1) & ~1;  // the loop body holds two steps (one per register set); an odd
                                    // count is padded with a step whose X and W read as zero

    u32x4 xfA[TM32], wfA[TN32], xfB[TM32], wfB[TN32];

    // One K step: MFMAs on stage kt % 2.  On entry `ws` holds W of step kt + 1, its first P3 pieces
    // already in the other stage; part 0 of the refill with X tile kt + 1 (into the other stage) and W
    // tile kt + 2 (into `wo`) has been issued.  Phases 0 and 1 issue the rest of it, phase 3 (after the
    // barrier, which vacates this stage, and after the last piece of `ws` has been staged) begins the
    // next refill: X tile kt + 2 into this stage, W tile kt + 3 into `ws`.
    auto k_step = [&](int kt, WSet& ws, WSet& wo) {
        const int cur = kt & 1;
        u32x4* a_cur = As + cur * A_SLOTS;
        u32x4* b_cur = Bs + cur * B_SLOTS;
        u32x4* a_nxt = As + (cur ^ 1) * A_SLOTS;
        u32x4* b_nxt = Bs + (cur ^ 1) * B_SLOTS;
#define IC(v) integral_constant<int, (v)> {}
        phase(IC(0), IC(1), IC(P3), IC(wp1 - P3), a_cur, b_cur, 1, xfA, wfA, xfB, wfB, a_nxt, kt + 1, wo, ws, b_nxt);
        phase(IC(1), IC(2), IC(wp1), IC(wp2 - wp1), a_cur, b_cur, 2, xfB, wfB, xfA, wfA, a_nxt, kt + 1, wo, ws, b_nxt);
        phase(IC(2), IC(-1), IC(wp2), IC(NP - wp2), a_cur, b_cur, 3, xfA, wfA, xfB, wfB, a_nxt, kt + 1, wo, ws, b_nxt);
        // The next tile is complete in LDS (the requests of its X part are followed by NWL younger
        // instructions only); nobody reads the current stage any more.
        stage_barrier(IC(NWL));
        phase(IC(3), IC(0), IC(0), IC(P3), a_nxt, b_nxt, 0, xfB, wfB, xfA, wfA, a_cur, kt + 2, ws, wo, b_cur);
#undef IC
    };

    // ---- prologue ----------------------------------------------------------------------------------
    // The global-memory instructions are issued in the order the loop issues them, so that the wait
    // counts computed for the loop body hold on entry as well: X 0, W 0, W 1, [stage W 0], part 0 of
    // the refill with X 1 and W 2.
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        request_x(As, 0, i);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
        load_w(ws_b, 0, i);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
        load_w(ws_a, 1, i);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) stage_w_piece(ws_b, Bs, p / (KR / 2), p % (KR / 2));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < MF; ++q) refill_slot(integral_constant<int, 0>{}, q, As + A_SLOTS, 1, ws_b);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < P3; ++p) stage_w_piece(ws_a, Bs + B_SLOTS, p / (KR / 2), p % (KR / 2));
    // X of tile 0 is older than everything but its own requests: 2 NWL + (NI + 2) / 3 younger instructions (part 0 of the refill) would do; the
    // prologue runs once, so it simply waits for everything (and does not depend on the order above).
    stage_barrier(integral_constant<int, 0>{});
    read_frags(As, Bs, 0, xfA, wfA);

    for (int kt = 0; kt < KT2; kt += 2) {
        k_step(kt, ws_a, ws_b);
        k_step(kt + 1, ws_b, ws_a);
    }

    // ---- 1/rms per row: four partial sums per row (two K halves of the operand x two wavefronts) ----
    // Requests past the last tile are still on their way to LDS (they deliver zeros).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // the stages are free: reuse the first one for the partials
    float* ss_part = (float*)As;  // [2 wn][2 lh][BM]
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) {
        const int sel = lane & 3;
        const float v = sel == 0 ? gram[ib][0] : sel == 1 ? gram[ib][1] : sel == 2 ? gram[ib][2] : gram[ib][3];
        ss_part[(wn * 2 + lh) * BM + wm * WTM + 32 * ib + l32] = v;
    }
    __syncthreads();
    if (tid < BM) {
        const float s = ss_part[tid] + ss_part[BM + tid] + ss_part[2 * BM + tid] + ss_part[3 * BM + tid];
        rscale[tid] = (flags & kFlagNorm) ? __builtin_amdgcn_rsqf(s / (float)K + eps) : 1.0f;
    }
    __syncthreads();

    // ---- epilogue: register v of block (jb, ib) is row 32 ib + l32, column 32 jb + 8 (v / 4) + 4 lh + v % 4.
    // A lane's 8 bytes of a row, stored from the registers, would be one cache request each (a quarter
    // of a million per tile, a tenth of everything the L2 sees, and the L2 is what this kernel keeps
    // busy).  So the finished tile goes through LDS, which is free now: every wavefront writes its own
    // part in the storage format and reads it back row by row, and a store instruction then covers
    // whole 64- to 256-byte runs of a row.  The staged row pitch is 8 bytes more than the row, which
    // spreads the 32 rows a store instruction touches over all banks.
    constexpr int OB = GATED ? TN32 / 2 : TN32;  // output 32-column blocks per wavefront
    constexpr int WOC = 32 * OB;                 // output columns per wavefront
    constexpr int PB = CW * 2 + 8;               // bytes per staged row
    constexpr int CPR = WOC / 8;                 // 16-byte pieces per row of a wavefront's part
    static_assert(BM * PB <= (2 * A_SLOTS + 2 * B_SLOTS) * 16, "the staged tile fits in the operand stages");
    static_assert((WTM * CPR) % 64 == 0, "whole store instructions");
    const bool act_silu = (flags & kFlagSilu) != 0;
    char* ostage = (char*)lds;
#pragma unroll
    for (int ib = 0; ib < TM32; ++ib) {
        const int ml = wm * WTM + 32 * ib + l32;
        const float r = rscale[ml];
#pragma unroll
        for (int jb = 0; jb < OB; ++jb) {
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int col = wn * WOC + 32 * jb + 4 * lh + 8 * vg;
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    y[e] = acc[jb][ib][4 * vg + e] * r;
                    if (GATED) y[e] = (act_silu ? silu_f32(y[e]) : y[e]) * (acc[jb + OB][ib][4 * vg + e] * r);
                }
                *(u32x2*)(ostage + ml * PB + col * 2) = u32x2{F::pack(y[0], y[1]), F::pack(y[2], y[3])};
            }
        }
    }
    // The same wavefront reads what it wrote (LDS accesses of a wavefront complete in order).
#pragma unroll
    for (int i = 0; i < WTM * CPR / 64; ++i) {
        const int idx = i * 64 + lane;
        const int row = idx / CPR, piece = idx % CPR;
        const int ml = wm * WTM + row;
        const int col = wn * WOC + 8 * piece;
        const u32x2 lo = *(const u32x2*)(ostage + ml * PB + col * 2);
        const u32x2 hi = *(const u32x2*)(ostage + ml * PB + col * 2 + 8);
        const int m = m0 + ml, n = n0 + col;
        if (m < M && n < N) *(u32x4*)(Y + (size_t)m * N + n) = u32x4{lo[0], lo[1], hi[0], hi[1]};
    }
}

template <typename F, int BM, int BN, bool GATED>
static hipError_t launch_tile(const Call& c) {
    constexpr int CW = GATED ? BN / 2 : BN;
    const int tiles_m = (c.M + BM - 1) / BM, tiles_n = (c.N + CW - 1) / CW;
    const size_t lds = (size_t)(2 * (BM / 8) * XGS + 2 * KCH * (BN + PAD)) * 16 + (size_t)BM * 4;
    auto kern = prefill_kernel<F, BM, BN, GATED>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), lds, c.stream, (const uint16_t*)c.X,
                       (const uint16_t*)c.g, (const uint16_t*)c.W1, (const uint16_t*)(c.gated ? c.W2 : c.W1),
                       (uint16_t*)c.Y, c.M, c.K, c.N, c.eps, tiles_m, tiles_n, c.flags);
    return hipGetLastError();
}

template <typename F>
static hipError_t launch_prefill_fmt(const Call& c, int tile_m, int tile_n) {
    if (c.gated) {
        if (tile_m == 256 && tile_n == 256) return launch_tile<F, 256, 256, true>(c);
        if (tile_m == 128 && tile_n == 256) return launch_tile<F, 128, 256, true>(c);
        if (tile_m == 128 && tile_n == 128) return launch_tile<F, 128, 128, true>(c);
    } else {
        if (tile_m == 256 && tile_n == 256) return launch_tile<F, 256, 256, false>(c);
        if (tile_m == 256 && tile_n == 192) return launch_tile<F, 256, 192, false>(c);
        if (tile_m == 256 && tile_n == 128) return launch_tile<F, 256, 128, false>(c);
        if (tile_m == 128 && tile_n == 128) return launch_tile<F, 128, 128, false>(c);
        if (tile_m == 64 && tile_n == 64) return launch_tile<F, 64, 64, false>(c);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_prefill_16bit(const Call& c, bool f16, int tile_m, int tile_n) {
    return f16 ? launch_prefill_fmt<F16>(c, tile_m, tile_n) : launch_prefill_fmt<Bf16>(c, tile_m, tile_n);
}

}  // namespace prism
