/*
 * prism.h - C ABI of the fused RMSNorm -> MatMul operator family for AMD MI355X (gfx950).
 *
 * The library computes, in one kernel launch and without ever writing the
 * normalised input to memory,
 *
 *     Y = rms_norm(X; g, eps) . W                            (prism_rmsnorm_matmul)
 *     Y = silu(rms_norm(X) . W1) * (rms_norm(X) . W2)        (prism_rmsnorm_gated_mlp)
 *
 * with rms_norm(X)[m,k] = X[m,k] * g[k] / sqrt(mean_k X[m,:]^2 + eps).
 *
 * These are the "RMSNorm", "RMSNorm-MLP" and "SwiGLU" workloads of the paper
 * (Section 7.1).  The kernels use the rewrite the paper's verifier licenses
 * (Table 1, "matmul commutes with div denominator"): the per-row sum of squares
 * is accumulated inside the GEMM K-loop and 1/rms is applied to the finished
 * accumulator, exactly as the running example's fused program accumulates its
 * row reduction in the loop and divides after it (Figure 1(b)).
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     allocates and frees nothing.  X, g, W* are only read; Y is overwritten and
 *     must not overlap any input.
 *   - g may be NULL: the call then has no gain tensor (g = 1), as in the paper's
 *     own workloads, whose rms_norm takes X alone (Section 7.1, Section 7.6).
 *   - Layout: row-major, contiguous.  X[M,K], g[K], W[K,N], Y[M,N].
 *   - dtype names the storage type of X, g, W*, Y alike.  PRISM_BF16 and PRISM_F16
 *     multiply on the matrix cores in that format and accumulate in fp32 (X * g is
 *     rounded to the format on its way in); PRISM_F32 uses fp32 FMAs.
 *   - Pointers must be 16-byte aligned.
 *   - Work is enqueued on `stream` and the call returns without waiting for it.
 *   - Errors are reported by return code only; nothing is printed or thrown.
 *     M == 0 or N == 0 returns PRISM_OK without a launch and without looking at the pointers.
 */
#ifndef PRISM_H
#define PRISM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Same opaque type as <hip/hip_runtime_api.h>; repeated so C callers need no HIP headers. */
typedef struct ihipStream_t* hipStream_t;

typedef enum {
    PRISM_OK = 0,
    PRISM_ERR_INVALID_ARG = 1, /* null or misaligned pointer, negative size, K == 0, eps < 0 or not finite */
    PRISM_ERR_UNSUPPORTED = 2, /* unknown dtype/op/path, or a forced path that cannot run this shape */
    PRISM_ERR_WORKSPACE = 3,   /* the chosen kernel needs a workspace and none (or too small a one) is set */
    PRISM_ERR_HIP = 4          /* the HIP runtime reported an error at launch */
} prism_status_t;

/* PRISM_F16 is the paper's own precision (Section 7.1: half precision). */
typedef enum { PRISM_F32 = 0, PRISM_BF16 = 1, PRISM_F16 = 2 } prism_dtype_t;

typedef enum {
    PRISM_OP_RMSNORM_MATMUL = 0,
    PRISM_OP_RMSNORM_GATED_MLP = 1, /* also prism_rmsnorm_glu and prism_swiglu */
    PRISM_OP_SOFTMAX_MATMUL = 2
} prism_op_t;

/* Kernel families.  AUTO picks by shape; the others are for tests and tuning sweeps. */
typedef enum {
    PRISM_PATH_AUTO = 0,
    PRISM_PATH_SIMPLE = 1,  /* plain FMA kernel: any M, K, N; the only path for PRISM_F32 */
    PRISM_PATH_DECODE = 2,  /* few rows: W streamed once, split-K over wavefronts and workgroups */
    PRISM_PATH_PREFILL = 3, /* many rows: LDS-tiled MFMA GEMM */
    PRISM_PATH_ROWS = 4,    /* prism_softmax_matmul only: the matrix-core kernels (variant 16: 16 rows of X over the
                               whole of K per workgroup; variant 32: 32 rows and one of up to 16 K-slices) */
    PRISM_PATH_ATTENTION = 5 /* prism_gqa_decode_attention only: matrix-core kernel, keys split over workgroups */
} prism_path_t;

/* What the dispatcher does for one call (filled by prism_plan). */
typedef struct {
    int32_t path;            /* prism_path_t actually used */
    int32_t split_k;         /* K-slices reduced across workgroups (1 = none) */
    int32_t tile_m, tile_n;  /* output tile of one workgroup */
    int32_t grid_x, grid_y;  /* launch grid */
    int32_t block;           /* threads per workgroup */
    int32_t grid_z;          /* launch grid, third dimension (0 or 1: none) */
    uint64_t workspace_bytes; /* workspace the call needs (0 = none) */
} prism_plan_t;

/*
 * Y[M,N] = rms_norm(X[M,K]; g[K], eps) . W[K,N]         (paper Section 7.1, workload "RMSNorm";
 * gain g and eps are this library's additions, see the conventions above; g = NULL and the
 * paper's operator is obtained).
 * Returns PRISM_OK once the work is enqueued.
 */
prism_status_t prism_rmsnorm_matmul(const void* X, const void* g, const void* W, void* Y,
                                    int64_t M, int64_t K, int64_t N, float eps,
                                    prism_dtype_t dtype, hipStream_t stream);

/*
 * Y[M,N] = silu(Nrm . W1) * (Nrm . W2),  Nrm = rms_norm(X; g, eps),  silu(a) = a / (1 + exp(-a)).
 * W1 is the gate branch (paper Section 7.1, workloads "RMSNorm-MLP" and "SwiGLU").
 * W1 and W2 are both [K,N].  The 1/rms scale is applied to both products before the activation.
 */
prism_status_t prism_rmsnorm_gated_mlp(const void* X, const void* g, const void* W1, const void* W2,
                                       void* Y, int64_t M, int64_t K, int64_t N, float eps,
                                       prism_dtype_t dtype, hipStream_t stream);

/*
 * The paper's "RMSNorm-MLP" workload exactly (Section 7.1): the two products that share the
 * normalised input, multiplied element by element, with no activation:
 * Y[M,N] = (Nrm . W1) * (Nrm . W2),  Nrm = rms_norm(X; g, eps).  Arguments as above.
 */
prism_status_t prism_rmsnorm_glu(const void* X, const void* g, const void* W1, const void* W2,
                                 void* Y, int64_t M, int64_t K, int64_t N, float eps,
                                 prism_dtype_t dtype, hipStream_t stream);

/*
 * The paper's "SwiGLU" workload exactly (Section 7.1): Y[M,N] = silu(X . W_gate) * (X . W_up),
 * no normalisation and no gain.  W_gate and W_up are both [K,N].
 */
prism_status_t prism_swiglu(const void* X, const void* W_gate, const void* W_up, void* Y,
                            int64_t M, int64_t K, int64_t N, prism_dtype_t dtype, hipStream_t stream);

/*
 * The paper's running example (Figure 1): Y[M,N] = softmax(X[M,K]) . W[K,N], the softmax taken
 * over k.  As in the fused program of Figure 1(b), exp and its row sum are accumulated in the loop
 * over k beside the product and the division follows the loop; softmax(X) is never written to
 * memory.  The row maximum is subtracted before the exponential (it cancels in exact arithmetic),
 * so any finite X is safe.  dtype as above.  Shapes whose plan splits K (prism_plan reports split_k > 1:
 * few rows against a deep K) hand partial results across workgroups through the workspace, like the
 * decode kernels: PRISM_ERR_WORKSPACE if prism_workspace_bytes(PRISM_OP_SOFTMAX_MATMUL, ...) is not met.
 */
prism_status_t prism_softmax_matmul(const void* X, const void* W, void* Y, int64_t M, int64_t K,
                                    int64_t N, prism_dtype_t dtype, hipStream_t stream);

/*
 * The paper's "Attention" and "QK-Attention" workloads (Section 7.1): group-query attention at one
 * query position,
 *     O[b,g,:] = softmax(scale * Qn[b,g,:] . K[b]^T) . V[b],
 * where the G query heads of batch entry b share its H keys and values, and Qn = rms_norm(Q) over
 * the head dimension D (no gain, eps inside the root) when qk_norm != 0, else Qn = Q.
 * Layouts (row-major, contiguous): Q[B,G,D], K[B,H,D], V[B,H,D], O[B,G,D].  The paper's formulas have
 * no 1/sqrt(D): scale = 1 is the paper's operator.  The softmax over the keys is never written to
 * memory.  When the keys are split over workgroups (prism_attention_workspace_bytes > 0) the call
 * needs the registered workspace, under the same rules as the split-K calls above.
 * prism_attention_plan reports path, slices (split_k), keys per slice (tile_n), grid and workspace.
 */
prism_status_t prism_gqa_decode_attention(const void* Q, const void* K, const void* V, void* O,
                                          int64_t B, int64_t G, int64_t H, int64_t D, float scale,
                                          int32_t qk_norm, float eps, prism_dtype_t dtype,
                                          hipStream_t stream);
uint64_t prism_attention_workspace_bytes(int64_t B, int64_t G, int64_t H, int64_t D, prism_dtype_t dtype);
prism_status_t prism_attention_plan(int64_t B, int64_t G, int64_t H, int64_t D, prism_dtype_t dtype,
                                    prism_plan_t* plan);

/* The first two operations with the storage type in the name instead of an argument. */
prism_status_t prism_rmsnorm_matmul_bf16(const void* X, const void* g, const void* W, void* Y,
                                         int64_t M, int64_t K, int64_t N, float eps, hipStream_t stream);
prism_status_t prism_rmsnorm_matmul_f32(const void* X, const void* g, const void* W, void* Y,
                                        int64_t M, int64_t K, int64_t N, float eps, hipStream_t stream);
prism_status_t prism_rmsnorm_gated_mlp_bf16(const void* X, const void* g, const void* W1, const void* W2,
                                            void* Y, int64_t M, int64_t K, int64_t N, float eps,
                                            hipStream_t stream);
prism_status_t prism_rmsnorm_gated_mlp_f32(const void* X, const void* g, const void* W1, const void* W2,
                                           void* Y, int64_t M, int64_t K, int64_t N, float eps,
                                           hipStream_t stream);

/*
 * Split-K workspace (paper Table 1, "parallelized matmul (reduction)": the K-slices of one
 * output tile are summed before the 1/rms scale and the activation).
 *
 * prism_workspace_bytes: bytes the given call needs under the current override (0 if none).
 * prism_set_workspace: registers caller-owned DEVICE memory (256-byte aligned) for the current
 *   HIP device.  The first PRISM_WORKSPACE_HEADER_BYTES hold per-tile arrival counters that
 *   must be zero between calls: this function zeroes them with a blocking hipMemset (the one
 *   place the library waits on the device) and every kernel leaves them zero again.  The
 *   memory must outlive all enqueued work.  Calls that use one workspace must not overlap in
 *   time (use one stream, or order the streams, or give streams workspaces of their own with
 *   prism_set_stream_workspace).  Passing NULL/0 unregisters.  The workspace belongs to the current HIP
 *   device, and a call finds it through the current device: call with the device of `stream` current.
 *   A kernel that fails after it has taken arrival tickets can leave counters non-zero: register the
 *   workspace again after any PRISM_ERR_HIP or device error before reusing it.
 * prism_set_stream_workspace: the same for calls on one stream: a call looks for a workspace registered for
 *   exactly its stream first and falls back to the device's.  With one workspace per stream, split-K calls on
 *   different streams may run at the same time.  At most 32 streams; NULL/0 unregisters the stream's.
 *   The calls themselves only enqueue kernels (no memset, no allocation, no synchronisation), so a
 *   sequence of them may be recorded in a HIP graph and replayed (tested).
 */
#define PRISM_WORKSPACE_HEADER_BYTES 262144u
uint64_t prism_workspace_bytes(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype);
prism_status_t prism_set_workspace(void* dev_ptr, uint64_t bytes);
prism_status_t prism_set_stream_workspace(hipStream_t stream, void* dev_ptr, uint64_t bytes);

/*
 * prism_rmsnorm_matmul for callers that cannot allocate or register device memory: code that is being recorded
 * into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-for-bit the same result as prism_rmsnorm_matmul, but a call whose plan splits K exchanges its partial sums
 * through an array of PRISM_STATIC_SCRATCH_BYTES that is part of the library's device code (every device the
 * library runs on holds it until the process ends) instead of the registered workspace.  The call allocates and
 * frees nothing and ignores prism_set_workspace.  The first call on a device looks the array's address up and
 * enqueues a small kernel on `stream` that clears its arrival counters; the current device must be the device of
 * `stream`.  PRISM_ERR_WORKSPACE if the call needs more than PRISM_STATIC_SCRATCH_BYTES
 * (prism_workspace_bytes tells; at most 16 rows against W[4096,4096] need 2.3 MB).  All calls on a device share the one
 * array: calls of this entry point that overlap in time on one device race (use one stream, or order the streams).
 */
#define PRISM_STATIC_SCRATCH_BYTES 8388608u
prism_status_t prism_rmsnorm_matmul_static(const void* X, const void* g, const void* W, void* Y,
                                           int64_t M, int64_t K, int64_t N, float eps,
                                           prism_dtype_t dtype, hipStream_t stream);

/*
 * Host-side query: fills *plan with the kernel family, split factor, tile and grid the
 * dispatcher would use for this shape under the current override.  Launches nothing; the first planning call of
 * a process asks the current device for its number of compute units (grids are sized by it; 256 is assumed where
 * there is no device to ask).
 */
prism_status_t prism_plan(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype,
                          prism_plan_t* plan);

/*
 * Process-wide override for tests and tuning: force a kernel family and/or a split-K factor and
 * a tile variant (0 = automatic for each).  Variants: PRISM_PATH_DECODE with at most 16 rows: 4, 8 or 16
 * wavefronts per workgroup, for gated calls also 104 and 108 (4 or 8 wavefronts, tiles of 64 output columns that
 * hold the products with W1 and with W2 in one matrix-core tile); with more rows: 32 or 64 rows per workgroup, or 36 / 68 for the same
 * row counts with X moved through LDS four K-blocks at a time (calls with one weight matrix only);
 * PRISM_PATH_PREFILL: 1000 * tile_m + tile_n; PRISM_PATH_ROWS: 16 or 32 rows per workgroup (a split applies
 * to 32 only, at most 16 slices).  A forced path that cannot run a shape makes the call
 * return PRISM_ERR_UNSUPPORTED.  The kernels are correct for every admissible value (the paper's
 * notion of a mapping that is correct for all parameter values, Section 2).
 */
prism_status_t prism_set_override(int32_t path, int32_t split_k, int32_t variant);

/*
 * Plan table: per-shape parameter assignments that take precedence over the built-in heuristic (but
 * not over prism_set_override).  This is where a tuner puts what it found: the paper instantiates
 * the parameters of a program by sampling valid assignments and profiling them (Section 5,
 * "parameter instantiation"); the kernels here are correct for every admissible assignment, so the
 * same can be done at run time (see the tune module of the Python package).
 * prism_plan_table_set: (path, split_k, variant) as in prism_set_override, for calls of exactly this
 *   (op, M, K, N, dtype); the three gated operations share PRISM_OP_RMSNORM_GATED_MLP.  Replaces an
 *   existing entry for the same key.  PRISM_ERR_UNSUPPORTED if the assignment cannot run the shape
 *   or the table (256 entries) is full.  Host-side only, thread-safe, touches no device.
 */
prism_status_t prism_plan_table_set(prism_op_t op, int64_t M, int64_t K, int64_t N, prism_dtype_t dtype,
                                    int32_t path, int32_t split_k, int32_t variant);
prism_status_t prism_plan_table_clear(void);
int32_t prism_plan_table_size(void);

/*
 * How the 16-row decode kernel deals K out to its workgroups (the reduction partition of paper Table 1,
 * "parallelized matmul (reduction)", with shares that are equal in streaming time instead of in K).
 *
 * Slow units.  When the row pitch of W is a multiple of 2 KiB, the stripe of W a workgroup streams keeps bits 7-10
 * of its byte addresses for all rows (which 128 bytes of every 2 KiB: its unit).  On the MI355X machines measured, the
 * stripes in units 3 and 11 arrive 40 % later than the others, wherever W starts and whichever CU reads them.
 * slow_units: bit u set = unit u is slow.  The default is 0 (none): which units are slow is a property of the
 * machine, to be measured there (the Python package's tune.detect_slow_units times the sixteen units with
 * prism_probe_units and returns the mask; 0x0808 on the machines measured, where it takes 3 % off the gated decode
 * configuration: 42.1 -> 40.7 us).  Used for gated calls with at most 16 rows:
 * they take tiles of 64 output columns (128-byte stripes of W1 and of W2) and cut the tiles in slow units into more
 * K-slices than the others, provided N is a multiple of 1024 and all workgroups find a CU of their own; the
 * balanced launch also needs W1 on a 128-byte boundary and W2 in step with W1 modulo 2 KiB (otherwise every tile gets
 * the same slices).  prism_plan then reports a one-dimensional grid, tile_n = 64 and, as split_k, the slices of a
 * slow tile (what the workspace is sized for).  The slices decide the order of the fp32 sums, so results may differ
 * in the last bit between buffers that start in different units; for given addresses they are reproducible.
 *
 * mode bit 0 (default off): for 129 to 159 column tiles, where one K-slice per tile leaves more than a third of the
 * CUs idle and two do not fit, launch 256 workgroups and give each the same share of all K-blocks, tile after tile;
 * a share may end one tile and begin the next (two passes).  prism_plan then reports a one-dimensional grid and,
 * as split_k, the most workgroups that can share a tile.  Off because three K-slices per tile, which the library
 * takes by default there, are faster on the MI355X measured.  mode bit 1 (default off): in that partition,
 * 256-byte-wide tiles that contain a slow unit weigh 5 : 4 (needs N a multiple of 1024 and W on a 256-byte
 * boundary).
 * Host-side, process-wide.
 */
prism_status_t prism_set_stream_balance(int32_t slow_units, int32_t mode);

const char* prism_status_string(prism_status_t status);
int32_t prism_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H */
