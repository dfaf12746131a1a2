/*
 * prism_diag.h - measurement and test hooks of libprism.  Not part of the operator boundary (prism.h): nothing here
 * computes a member of the operator family.  bench.py and the tests use these entry points.
 */
#ifndef PRISM_DIAG_H
#define PRISM_DIAG_H

#include "prism.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostic, host-side: the K-blocks [*first, *first + *count) of column tile `tile` that workgroup `wg` works on
 * in a weighted partition of n_tiles tiles of kblocks K-blocks over `workgroups` workgroups; a K-block of tile t
 * weighs w_slow if bit (t mod period) of slow_tiles is set, else w_fast (period 8 or 16).  The same integer
 * functions run in the kernel; this entry point lets a test check that they deal every K-block out exactly once.
 * PRISM_ERR_UNSUPPORTED if the total weight does not fit 31 bits.
 */
prism_status_t prism_stream_partition_blocks(int32_t workgroups, int32_t kblocks, int32_t n_tiles, int32_t slow_tiles,
                                            int32_t period, int32_t w_fast, int32_t w_slow, int32_t wg, int32_t tile,
                                            int32_t* first, int32_t* count);

/*
 * Diagnostic, for measurement: streams W[K,N] (16-bit elements, device memory, 16-byte aligned, N a multiple
 * of 8; and W2 of the same shape unless NULL) once with the decode kernels' access pattern and split, and
 * computes nothing.  Its duration is the
 * floor that streaming W sets for a decode call on the machine at hand (bench.py reports it beside the
 * kernels).  Needs a registered workspace of at least 2 * PRISM_WORKSPACE_HEADER_BYTES (one word past the
 * counters may be written).
 */
prism_status_t prism_probe_stream(const void* W, const void* W2, int64_t K, int64_t N, int32_t split_k,
                                  hipStream_t stream);

/*
 * For measurement: 16 * groups workgroups read [base, base + bytes) (device memory, 2 KiB aligned) once, all at the
 * same time; the buffer is cut into `groups` equal runs of 2 KiB blocks, and workgroup j reads, of every block of run
 * j / 16, the 128 bytes at offset 128 * (j % 16) - one of the sixteen address units - and computes nothing.  A stripe
 * of a matrix whose row pitch is a multiple of 2 KiB looks like this to the memory system.  ticks[j] (device memory,
 * 16 * groups words of 8 bytes) receives workgroup j's duration in ticks of the 100 MHz real-time counter: units that
 * stream slowly while the others are busy too show up as longer times (prism_set_stream_balance takes the mask).
 * A run must stay below 2 GiB.
 */
prism_status_t prism_probe_units(const void* base, uint64_t bytes, int32_t groups, uint64_t* ticks, hipStream_t stream);

/*
 * For measurement: what one compute unit's vector-memory path delivers for a given shape of load instruction on data
 * that stays in the L2.  `workgroups` workgroups of eight wavefronts each read the first PRISM_PROBE_LOADS_BYTES of
 * [base, base + bytes) (device memory, 16-byte aligned; 128 rows of 8 KiB) `reps` times, eight loads in flight per
 * lane, and compute nothing.  pattern 0: four rows x 256 contiguous bytes per instruction (how the decode kernels
 * read W); 1: sixteen rows x 64 bytes (an MFMA A operand read straight from a row-major matrix); 2: eight rows x
 * 128 bytes; 3: four rows x 128 bytes with 8-byte loads.  ticks (device memory, 8 * workgroups words of 8 bytes)
 * receives the shader-clock cycles of every wavefront; a workgroup moves reps * 1 MiB (pattern 3: half of that).
 */
#define PRISM_PROBE_LOADS_BYTES 1048576u
prism_status_t prism_probe_loads(const void* base, uint64_t bytes, int32_t pattern, int32_t reps, int32_t workgroups,
                                 uint64_t* ticks, hipStream_t stream);

/*
 * For measurement: reads [base, base + bytes) (device memory, 16-byte aligned, bytes a multiple of 16) once, front to
 * back: workgroup j of `workgroups` streams the j-th contiguous piece and computes nothing.  The same bytes as a
 * weight matrix without any stripe structure: a second opinion on what streaming them costs.  sink: 4 bytes of
 * device memory (one word may be written).
 */
prism_status_t prism_probe_linear(const void* base, uint64_t bytes, int32_t workgroups, void* sink, hipStream_t stream);

/*
 * For measurement: `workgroups` workgroups of four wavefronts issue 16 * iters 32x32x16 bf16 MFMAs each on
 * registers, with no memory or LDS traffic: 32768 * 16 * iters * 4 * workgroups flops.  What the matrix pipes
 * sustain on the machine at hand (clock and power limit included): the measured ceiling beside the published peak.
 * sink: 4 bytes of device memory (never written in practice).
 */
prism_status_t prism_probe_mfma(void* sink, int32_t workgroups, int32_t iters, hipStream_t stream);

/*
 * The planner sizes grids by the number of compute units of the current device (asked once; 256 where no device
 * can be asked).  prism_diag_set_cu_count(n) makes it plan for n units instead (0: back to the device's count), so
 * that tests can check the plans for other parts or partition modes on any host.  prism_diag_cu_count: the count
 * in use.
 */
prism_status_t prism_diag_set_cu_count(int32_t cus);
int32_t prism_diag_cu_count(void);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_DIAG_H */
