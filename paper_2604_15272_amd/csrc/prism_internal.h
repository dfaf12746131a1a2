// Internal declarations shared by the C-ABI file and the kernel files (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "prism.h"
#include "prism_diag.h"

namespace prism {

struct Call {
    const void* X;
    const void* g;
    const void* W1;
    const void* W2;  // null unless gated
    void* Y;
    int M, K, N;
    float eps;
    bool gated;
    int flags;  // kFlag* bits
    hipStream_t stream;
};

// Members of the operator family (paper Section 7.1): which of the optional steps a call takes.
constexpr int kFlagGain = 1;  // multiply the row by g[K] (off: g is not read)
constexpr int kFlagNorm = 2;  // scale by 1/rms (off: the sums of squares are ignored)
constexpr int kFlagSilu = 4;  // gated calls: SiLU on the W1 branch (off: plain product of the branches)

struct SoftmaxCall {
    const void* X;
    const void* W;
    void* Y;
    int M, K, N;
    hipStream_t stream;
};

struct AttentionCall {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    int B, G, H, D;
    float scale;
    int qk_norm;
    float eps;
    hipStream_t stream;
};

// The matrix-core attention kernel: head dimension, rows (query heads) per batch entry, key slices.
constexpr int kAttnHeadDim = 128;
constexpr int kAttnMaxHeads = 16;
constexpr int kAttnSliceKeys = 128;     // keys per workgroup for short contexts (one 32-key block per wavefront)
constexpr int kAttnMaxSlices = 64;

struct AttentionPlan {
    int path;        // PRISM_PATH_SIMPLE or PRISM_PATH_ATTENTION
    int splits;      // key slices per batch entry
    int slice_keys;  // keys per slice (a multiple of 32)
    uint64_t workspace_bytes;
};

struct AttentionWorkspace {
    unsigned* tickets;  // [B], in the workspace header, zero between calls
    float* m_part;      // [B][S][16]
    float* l_part;      // [B][S][16]
    float* acc_part;    // [B][S][16][128]
};

// Geometry of the softmax kernel: rows of X and columns of W per workgroup.
constexpr int kSoftmaxRows = 16;
constexpr int kSoftmaxTileN = 128;
// The K-split softmax kernel: rows per workgroup and most K-slices.
constexpr int kSoftmaxSplitRows = 32;
constexpr int kSoftmaxMaxSplits = 16;

struct SoftmaxWorkspace {
    unsigned* tickets;  // [row_blocks][n_tiles], in the workspace header, zero between calls
    float* ml_part;     // [row_blocks][n_tiles][S][32 rows][2]: slice maximum and sum of exponentials
    float* acc_part;    // [S][M][N] partial products
};

// Geometry of the decode (few-row) path.
constexpr int kDecodeMaxRows = 16;     // one 16-row MFMA block (the 16-row kernel)
// More rows than that still take the decode path (its multi-row-group kernel) up to this count, shape
// permitting; beyond it re-reading W per row block costs more than the tiled prefill kernel.
constexpr int kDecodeRowsMax = 512;
constexpr int kDecodeTileN = 128;      // columns of W per workgroup
constexpr int kDecodeKBlock = 32;      // K depth of one MFMA
constexpr int kDecodeWaves = 8;        // wavefronts per workgroup (default variant)
constexpr int kMaxTickets = PRISM_WORKSPACE_HEADER_BYTES / 4;

struct DecodeWorkspace {
    unsigned* tickets;  // [row_blocks][n_tiles] arrival counters, zero between calls
    float* ss_part;     // [row_blocks][n_tiles][S][rows per workgroup] partial sums of squares
    float* acc_part;    // [S][G][M][N] partial products (G = 2 if gated)
};

// Kernels with more than 64 KiB of dynamic LDS must be opted in once per device; `done` remembers
// which devices (bit = ordinal) have been.
inline hipError_t allow_large_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
    if (bytes <= 65536) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_relaxed) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_relaxed);
    return e;
}

hipError_t launch_simple_f32(const Call& c);
hipError_t launch_simple_bf16(const Call& c);
hipError_t launch_simple_f16(const Call& c);
// The matrix-core kernels, for either 16-bit storage format (f16 = false: bf16).
struct StreamPartition;
hipError_t launch_decode_16bit(const Call& c, bool f16, int split_k, const StreamPartition& sp, int waves, bool packed,
                               const DecodeWorkspace& ws);
hipError_t launch_decode_rows_16bit(const Call& c, bool f16, int split_k, int row_groups, bool xlds,
                                    const DecodeWorkspace& ws);
hipError_t launch_prefill_16bit(const Call& c, bool f16, int tile_m, int tile_n);
hipError_t launch_softmax_rows_16bit(const SoftmaxCall& c, bool f16);
hipError_t launch_softmax_split_16bit(const SoftmaxCall& c, bool f16, int split_k, const SoftmaxWorkspace& ws);
hipError_t launch_probe_stream(const void* W, const void* W2, unsigned* sink, int K, int N, int S, hipStream_t stream);
hipError_t launch_probe_units(const void* base, unsigned blocks_per_group, int groups, unsigned long long* ticks,
                              hipStream_t stream);
hipError_t launch_probe_loads(const void* base, int pattern, int reps, int workgroups, unsigned long long* ticks,
                              hipStream_t stream);
hipError_t launch_probe_linear(const void* base, unsigned long long bytes, int workgroups, unsigned* sink, hipStream_t stream);
hipError_t launch_probe_mfma(float* sink, int workgroups, int iters, hipStream_t stream);
hipError_t launch_softmax_simple(const SoftmaxCall& c, int dtype);
hipError_t launch_gqa_16bit(const AttentionCall& c, bool f16, const AttentionPlan& p, const AttentionWorkspace& ws);
hipError_t launch_gqa_simple(const AttentionCall& c, int dtype);

}  // namespace prism
