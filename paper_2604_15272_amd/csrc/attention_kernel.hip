// Group-query attention at one query position (paper Section 7.1, workloads "Attention" and
// "QK-Attention"):  O[b,g,:] = softmax(scale * Qn[b,g,:] . K[b]^T) . V[b],  Qn = rms_norm(Q) over the
// head dimension when qk_norm is set, else Q.  G query heads share the keys and values of their
// batch entry, so per batch entry this is a G x D by D x H product, a softmax over H, and a G x H
// by H x D product: the softmax -> matmul of the running example with its input computed on the
// fly, and with few rows, so the work is split over the keys instead (paper Table 1, the
// reduction partition of a matmul, here with the maximum and the sum of the softmax travelling
// with the partial product).
//
// Matrix-core kernel (16-bit storage, D = 128, G <= 16): a workgroup of four wavefronts owns one
// batch entry and one slice of the keys; a wavefront takes the slice's 32-key blocks round-robin and
// runs its own softmax over them, so nothing is synchronised until the partial outputs meet.
//   1. scores: K is D-contiguous, which is the layout of an MFMA B operand (8 head-dimension
//      values per lane), so a lane loads its operand of key c straight from memory; Q as stored is the
//      A operand, rows padded to 16.  The scale and, for QK-Attention, 1/rms of the head are applied
//      to the scores, not to Q (the paper's rewrite: the division by the norm commutes with the
//      matmul, Table 1).
//   2. per head: running maximum over the wavefront's blocks (accumulators rescaled when it moves), exp,
//      rounding to the storage format, sum of the rounded values; all in the registers the scores landed in.
//   3. values: the rounded 16 x 32 tile of P goes through the wavefront's own piece of LDS into A-operand
//      layout; a 32 x 128 block of V is turned into B operands as in the decode kernel (8 x 8 sub-blocks,
//      byte permutes).  The wavefronts' partial outputs, each relative to its own maximum, meet in LDS.
//   4. slices: each stores (partial output, maximum, sum) with device-coherent stores, waits for
//      the acknowledgement and takes a ticket; the last arrival of a batch entry rescales and adds
//      the partials in slice order, divides and stores O.  With one slice the division is direct.
// Everything is tiny at the paper's sizes (1 - 2 MiB of keys and values in all): the kernel is bound
// by its chain of dependent steps, not by bandwidth.
//
// Plain kernel: any head dimension up to 1024, any G, any storage type; one workgroup per (head,
// batch entry), keys in chunks of 256 with a running maximum.
#include <type_traits>

#include "device_utils.h"
#include "exchange.h"
#include "prism_internal.h"
#include "w_block.h"

namespace prism {

namespace {

constexpr int AD = kAttnHeadDim;  // 128
constexpr int ANW = 4;            // wavefronts per workgroup
constexpr float kLog2e = 1.4426950408889634f;

template <typename T> __device__ __forceinline__ float at_ld(const T* p, size_t i);
template <> __device__ __forceinline__ float at_ld<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float at_ld<uint16_t>(const uint16_t* p, size_t i) {
    return __builtin_bit_cast(float, (u32)p[i] << 16);
}
template <> __device__ __forceinline__ float at_ld<_Float16>(const _Float16* p, size_t i) { return (float)p[i]; }
template <typename T> __device__ __forceinline__ void at_st(T* p, size_t i, float v);
template <> __device__ __forceinline__ void at_st<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void at_st<uint16_t>(uint16_t* p, size_t i, float v) {
    p[i] = (uint16_t)(pack_bf16(v, 0.0f) & 0xFFFFu);
}
template <> __device__ __forceinline__ void at_st<_Float16>(_Float16* p, size_t i, float v) { p[i] = (_Float16)v; }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace

// ---- matrix-core kernel --------------------------------------------------------------------------
// Workspace (S > 1): acc_part[B][S][16][128] fp32, m_part[B][S][16], l_part[B][S][16], tickets[B].
template <typename F>
__global__ __launch_bounds__(ANW * 64) void gqa_decode_kernel(const uint16_t* __restrict__ Q,
                                                              const uint16_t* __restrict__ K,
                                                              const uint16_t* __restrict__ V,
                                                              uint16_t* __restrict__ O, float* __restrict__ acc_part,
                                                              float* __restrict__ m_part, float* __restrict__ l_part,
                                                              unsigned* __restrict__ tickets, int G, int H, int S,
                                                              int slice_keys, float scale, int qk_norm, float eps) {
    constexpr int NT = ANW * 64;
    constexpr int CPT = 16 * AD / NT;  // 8 output columns per thread
    constexpr int TPR = AD / CPT;      // 16 threads per output row
    const int KS = slice_keys;         // keys per slice, a multiple of 32
    constexpr int PW = 40;             // row pitch (elements) of a wavefront's 16 x 32 tile of P: rows 80 bytes apart

    extern __shared__ __align__(16) float lds[];  // 16-byte LDS accesses need the alignment said
    float* red = lds;                                   // [ANW][16][AD] partial outputs
    float* wm = red + ANW * 16 * AD;                    // [ANW][16] running maxima of the wavefronts
    float* wl = wm + ANW * 16;                          // [ANW][16] their sums of exponentials
    uint16_t* pr = (uint16_t*)(wl + ANW * 16);          // [ANW][16][PW] exp(score - max), storage format
    __shared__ int is_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane >> 4, c = lane & 15;
    const int s = blockIdx.x, bi = blockIdx.y;
    const int key0 = s * KS;
    const int nkeys = min(KS, H - key0);          // > 0: the host never launches an empty slice
    const int nblk = (nkeys + 31) / 32;

    const __amdgpu_buffer_rsrc_t rq = make_rsrc(Q + (size_t)bi * G * AD, (u32)(G * AD * 2));
    const __amdgpu_buffer_rsrc_t rk = make_rsrc(K + (size_t)bi * H * AD, (u32)((size_t)H * AD * 2));
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(V + (size_t)bi * H * AD, (u32)((size_t)H * AD * 2));

    // ---- Q as A operands of the four 32-deep blocks of the head dimension; lane (q, c): head c.
    u32x4 a_q[4];
    float f4[4];  // factor applied to the scores of heads 4q .. 4q+3 (the rows this lane holds of a score block)
    {
        float ss = 0.f;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            a_q[kb] = load16(rq, c < G ? (u32)((c * AD + 32 * kb + 8 * q) * 2) : kOutOfRange);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float x0 = F::lo(a_q[kb][d]), x1 = F::hi(a_q[kb][d]);
                ss = fmaf(x0, x0, ss);
                ss = fmaf(x1, x1, ss);
            }
        }
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        // The factor of a head (scale, times 1/rms when Q is normalised) goes on after the product with
        // K (paper Table 1, "matmul commutes with div denominator"): Q enters the matrix core as stored, with
        // no second rounding, and the sums of squares ride along the operand loads.
        const float f_c = qk_norm ? scale * __builtin_amdgcn_rsqf(ss / (float)AD + eps) : scale;  // head c
#pragma unroll
        for (int i = 0; i < 4; ++i) f4[i] = __shfl(f_c, 4 * q + i, 64);
    }

    // The V block of this wavefront's first key block is requested now, before its scores are computed.
    WRows w_first;
    const u32 v_lane = (u32)(((size_t)(key0 + 8 * q) * AD) * 2 + 16 * c);
    load_w_block<true>(w_first, rv, wave < nblk ? v_lane + (u32)(32 * wave * AD * 2) : kOutOfRange, (u32)(AD * 2));

    // ---- A wavefront takes the slice's 32-key blocks round-robin and runs its own softmax over them: scores on
    // the matrix cores (element i of a block in lane (q, c): head 4q + i, key c), a running maximum per head
    // with the accumulators rescaled when it moves, exp and rounding, the rounded tile through the wavefront's
    // own piece of LDS into operand layout (head c, keys 8q .. 8q+7), then P . V.  No barrier until the
    // wavefronts' partials meet.
    float m_run[4], l_run[4];
    f32x4 acc[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { m_run[i] = -__builtin_inff(); l_run[i] = 0.f; }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint16_t* pw = pr + wave * 16 * PW;
    for (int jb = wave; jb < nblk; jb += ANW) {
        u32x4 kf[2][4];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int key = key0 + 32 * jb + 16 * half + c;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
                kf[half][kb] = load16_stream(rk, key < H ? (u32)(((size_t)key * AD + 32 * kb + 8 * q) * 2) : kOutOfRange);
        }
        WRows w = w_first;
        if (jb != wave) load_w_block<true>(w, rv, v_lane + (u32)(32 * jb * AD * 2), (u32)(AD * 2));
        float sc[2][4];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            f32x4 t = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) t = F::mfma_16x16x32(a_q[kb], kf[half][kb], t);
            const bool valid = key0 + 32 * jb + 16 * half + c < H;
#pragma unroll
            for (int i = 0; i < 4; ++i) sc[half][i] = valid ? t[i] * f4[i] : -__builtin_inff();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float mb = fmaxf(sc[0][i], sc[1][i]);
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) mb = fmaxf(mb, __shfl_xor(mb, off, 64));
            const float m_new = fmaxf(m_run[i], mb);
            // nothing accumulated yet: factor 1 (and no -inf minus -inf)
            const float fac = (m_run[i] == -__builtin_inff()) ? 1.0f : __builtin_amdgcn_exp2f((m_run[i] - m_new) * kLog2e);
            m_run[i] = m_new;
            l_run[i] *= fac;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j][i] *= fac;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const float x = sc[half][i];
                const float e = (x == -__builtin_inff()) ? 0.f : __builtin_amdgcn_exp2f((x - m_new) * kLog2e);
                const u32 packed = F::pack(e, 0.f);
                l_run[i] += F::lo(packed);  // the sum weighs what the product will see: the rounded value
                pw[(4 * q + i) * PW + 16 * half + c] = (uint16_t)(packed & 0xFFFFu);
            }
        }
        // The wavefront reads what it wrote (its LDS accesses complete in order).
        const u32x4 a = *(const u32x4*)(pw + c * PW + 8 * q);
        acc[0] = F::mfma_16x16x32(a, b_operand<0>(w), acc[0]);
        acc[1] = F::mfma_16x16x32(a, b_operand<1>(w), acc[1]);
        acc[2] = F::mfma_16x16x32(a, b_operand<2>(w), acc[2]);
        acc[3] = F::mfma_16x16x32(a, b_operand<3>(w), acc[3]);
        acc[4] = F::mfma_16x16x32(a, b_operand<4>(w), acc[4]);
        acc[5] = F::mfma_16x16x32(a, b_operand<5>(w), acc[5]);
        acc[6] = F::mfma_16x16x32(a, b_operand<6>(w), acc[6]);
        acc[7] = F::mfma_16x16x32(a, b_operand<7>(w), acc[7]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) l_run[i] += __shfl_xor(l_run[i], off, 64);
        if (c == 0) {
            wm[wave * 16 + 4 * q + i] = m_run[i];
            wl[wave * 16 + 4 * q + i] = l_run[i];
        }
    }

    // ---- across wavefronts through LDS: each partial is relative to its wavefront's maximum.  Accumulator j,
    // element i of lane (q, c) is head 4q + i, column 8c + j.
    // Rows from G on are padding: the lanes that hold only such rows store nothing, the threads that would
    // combine them have nothing to do until the end.
    if (4 * q < G) store_acc_tile(red + wave * 16 * AD, AD, q, c, acc);
    __syncthreads();
    const int m = tid / TPR;           // head
    const int col = (tid % TPR) * CPT; // first of 8 output columns
    const bool head_ok = m < G;
    float row_max = -__builtin_inff();
    float v[CPT], den = 0.f;
#pragma unroll
    for (int e = 0; e < CPT; ++e) v[e] = 0.f;
    if (head_ok) {
#pragma unroll
        for (int w = 0; w < ANW; ++w) row_max = fmaxf(row_max, wm[w * 16 + m]);
#pragma unroll
        for (int w = 0; w < ANW; ++w) {
            const float mw = wm[w * 16 + m];
            const float fw = (mw == -__builtin_inff()) ? 0.f : __builtin_amdgcn_exp2f((mw - row_max) * kLog2e);  // a wavefront without keys
            const float* src = red + (w * 16 + m) * AD + col;
#pragma unroll
            for (int e = 0; e < CPT; ++e) v[e] = fmaf(fw, src[e], v[e]);
            den = fmaf(fw, wl[w * 16 + m], den);
        }
    }

    // ---- 4. across the slices of this batch entry
    if (S > 1) {
        const __amdgpu_buffer_rsrc_t racc = exchange_rsrc(acc_part, (size_t)gridDim.y * S * 16 * AD);
        if (head_ok) {
            store_partial<CPT>(racc, acc_part, (((size_t)bi * S + s) * 16 + m) * AD + col, v);
            if (col == 0) {
                store_coherent(m_part + ((size_t)bi * S + s) * 16 + m, row_max);
                store_coherent(l_part + ((size_t)bi * S + s) * 16 + m, den);
            }
        }
        wait_stores_acknowledged();
        __syncthreads();
        if (tid == 0) {
            const unsigned prev = __hip_atomic_fetch_add(&tickets[bi], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (prev == (unsigned)(S - 1));
        }
        __syncthreads();
        if (!is_last) return;
        if (tid == 0) tickets[bi] = 0u;  // ready for the next call on this workspace
        // Global maximum of the row, then the partials rescaled by exp(m_s - max), in slice order.  Eight
        // slices' loads are issued before the first is used (one round trip to memory per batch, not per slice;
        // sixteen at a time spill registers and double the kernel's time).  With eight slices or fewer the
        // maximum comes out of the same batch (one round trip in all); with more, all slices' maxima are read
        // first, in one round trip: the workgroup's threads share the (slice, head) pairs and pass them on
        // through LDS (the partial outputs there have been consumed before the barriers above).
        constexpr int BATCH = 8;
        float gmax = -__builtin_inff();
        if (S > BATCH) {
            float* sm = red;  // [S][16]
            constexpr int PER = kAttnMaxSlices * 16 / NT;
            float mv[PER];
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int idx = tid + NT * k;
                mv[k] = idx < S * 16 ? load_coherent(m_part + (size_t)bi * S * 16 + idx) : -__builtin_inff();
            }
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int idx = tid + NT * k;
                if (idx < S * 16) sm[idx] = mv[k];
            }
            __syncthreads();
            if (head_ok)
                for (int t = 0; t < S; ++t) gmax = fmaxf(gmax, sm[t * 16 + m]);
        }
        if (!head_ok) return;
#pragma unroll
        for (int e = 0; e < CPT; ++e) v[e] = 0.f;
        den = 0.f;
        for (int t0 = 0; t0 < S; t0 += BATCH) {
            float mm[BATCH], ll[BATCH];
            float x[BATCH][CPT];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const size_t row = ((size_t)bi * S + min(t0 + j, S - 1)) * 16 + m;  // slots past the last slice re-read it
                mm[j] = load_coherent(m_part + row);
                ll[j] = load_coherent(l_part + row);
                load_partial<CPT>(racc, acc_part, row * AD + col, x[j]);
            }
            if (S <= BATCH) {
#pragma unroll
                for (int j = 0; j < BATCH; ++j) gmax = fmaxf(gmax, mm[j]);  // slots past the last slice repeat it
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                if (t0 + j >= S) break;
                const float w = __builtin_amdgcn_exp2f((mm[j] - gmax) * kLog2e);
                den = fmaf(ll[j], w, den);
#pragma unroll
                for (int e = 0; e < CPT; ++e) v[e] = fmaf(x[j][e], w, v[e]);
            }
        }
    }
    if (m >= G) return;
    const float inv = 1.0f / den;
    const u32x4 out = u32x4{F::pack(v[0] * inv, v[1] * inv), F::pack(v[2] * inv, v[3] * inv),
                            F::pack(v[4] * inv, v[5] * inv), F::pack(v[6] * inv, v[7] * inv)};
    *(u32x4*)(O + ((size_t)bi * G + m) * AD + col) = out;
}

// Partial outputs, maxima and sums of the wavefronts, and their 16 x 32 tiles of P (row pitch 40 elements).
constexpr size_t kAttentionLdsBytes = (size_t)(ANW * 16 * AD + 2 * ANW * 16) * 4 + (size_t)ANW * 16 * 40 * 2;

template <typename F>
static hipError_t launch_gqa_fmt(const AttentionCall& c, const AttentionPlan& p, const AttentionWorkspace& ws) {
    dim3 grid(p.splits, c.B), block(ANW * 64);
    const size_t lds = kAttentionLdsBytes;
    auto kern = gqa_decode_kernel<F>;
    static std::atomic<uint64_t> opted{0};
    if (hipError_t e = allow_large_lds((const void*)kern, lds, opted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, c.stream, (const uint16_t*)c.Q, (const uint16_t*)c.K,
                       (const uint16_t*)c.V, (uint16_t*)c.O, ws.acc_part, ws.m_part, ws.l_part, ws.tickets, c.G, c.H,
                       p.splits, p.slice_keys, c.scale, c.qk_norm, c.eps);
    return hipGetLastError();
}

hipError_t launch_gqa_16bit(const AttentionCall& c, bool f16, const AttentionPlan& p, const AttentionWorkspace& ws) {
    return f16 ? launch_gqa_fmt<F16>(c, p, ws) : launch_gqa_fmt<Bf16>(c, p, ws);
}

// ---- plain kernel -----------------------------------------------------------------------------------
constexpr int kAtThreads = 256;
constexpr int kAtColsPerThread = 4;  // head dimension up to 1024

template <typename T>
__global__ __launch_bounds__(kAtThreads) void gqa_simple_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                                                               const T* __restrict__ V, T* __restrict__ O, int G, int H,
                                                               int D, float scale, int qk_norm, float eps) {
    __shared__ float qs[kAtThreads * kAtColsPerThread];
    __shared__ float pbuf[kAtThreads];
    __shared__ float part[kAtThreads / 64];
    __shared__ float bcast;
    const int t = threadIdx.x, g = blockIdx.x, bi = blockIdx.y;
    const T* q = Q + ((size_t)bi * G + g) * D;
    const T* kb = K + (size_t)bi * H * D;
    const T* vb = V + (size_t)bi * H * D;

    // Q (normalised if asked, scaled) in LDS as fp32
    float ss = 0.f;
    for (int d = t; d < D; d += kAtThreads) {
        const float x = at_ld<T>(q, d);
        qs[d] = x;
        ss = fmaf(x, x, ss);
    }
    ss = wave_sum(ss);
    if ((t & 63) == 0) part[t >> 6] = ss;
    __syncthreads();
    if (t == 0) {
        float tot = 0.f;
        for (int w = 0; w < kAtThreads / 64; ++w) tot += part[w];
        bcast = qk_norm ? scale / sqrtf(tot / (float)D + eps) : scale;
    }
    __syncthreads();
    const float f = bcast;
    for (int d = t; d < D; d += kAtThreads) qs[d] *= f;
    __syncthreads();

    float run_max = -__builtin_inff(), run_sum = 0.f;
    float acc[kAtColsPerThread];
#pragma unroll
    for (int j = 0; j < kAtColsPerThread; ++j) acc[j] = 0.f;
    for (int k0 = 0; k0 < H; k0 += kAtThreads) {
        // one key per thread: its score
        const int key = k0 + t;
        float sv = -__builtin_inff();
        if (key < H) {
            sv = 0.f;
            for (int d = 0; d < D; ++d) sv = fmaf(qs[d], at_ld<T>(kb, (size_t)key * D + d), sv);
        }
        float cm = wave_max(sv);
        __syncthreads();  // pbuf and part of the previous chunk are no longer read
        if ((t & 63) == 0) part[t >> 6] = cm;
        __syncthreads();
        cm = part[0];
#pragma unroll
        for (int w = 1; w < kAtThreads / 64; ++w) cm = fmaxf(cm, part[w]);
        const float new_max = fmaxf(run_max, cm);
        const float alpha = expf(run_max - new_max);  // 0 for the first chunk
        const float e = (key < H) ? expf(sv - new_max) : 0.f;
        pbuf[t] = e;
        float cs = wave_sum(e);
        __syncthreads();  // part (maxima) consumed by everyone; pbuf written
        if ((t & 63) == 0) part[t >> 6] = cs;
        __syncthreads();
        float csum = 0.f;
#pragma unroll
        for (int w = 0; w < kAtThreads / 64; ++w) csum += part[w];
        run_sum = run_sum * alpha + csum;
        run_max = new_max;
        const int kn = min(kAtThreads, H - k0);
#pragma unroll
        for (int j = 0; j < kAtColsPerThread; ++j) {
            const int d = t + j * kAtThreads;
            if (d < D) {
                float a = acc[j] * alpha;
                for (int kk = 0; kk < kn; ++kk) a = fmaf(pbuf[kk], at_ld<T>(vb, (size_t)(k0 + kk) * D + d), a);
                acc[j] = a;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kAtColsPerThread; ++j) {
        const int d = t + j * kAtThreads;
        if (d < D) at_st<T>(O, ((size_t)bi * G + g) * D + d, acc[j] / run_sum);
    }
}

template <typename T>
static hipError_t launch_gqa_simple_t(const AttentionCall& c) {
    dim3 grid(c.G, c.B), block(kAtThreads);
    hipLaunchKernelGGL((gqa_simple_kernel<T>), grid, block, 0, c.stream, (const T*)c.Q, (const T*)c.K, (const T*)c.V,
                       (T*)c.O, c.G, c.H, c.D, c.scale, c.qk_norm, c.eps);
    return hipGetLastError();
}

hipError_t launch_gqa_simple(const AttentionCall& c, int dtype) {
    if (dtype == PRISM_F32) return launch_gqa_simple_t<float>(c);
    if (dtype == PRISM_F16) return launch_gqa_simple_t<_Float16>(c);
    return launch_gqa_simple_t<uint16_t>(c);
}

}  // namespace prism
