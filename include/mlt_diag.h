/*
 * mlt_diag.h: diagnostics of the mlt library: measurement probes, per-kernel timing hooks, the
 * name and tiling of the kernel a call selects, and overrides of that selection. None of this is
 * part of the operations declared in mlt.h; benchmarks and tests use it. Conventions (device
 * pointers, streams, status codes) as in mlt.h.
 */
#ifndef MLT_DIAG_H_
#define MLT_DIAG_H_

#include "mlt.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostic for benchmarks (not part of the paper's method): enqueues one kernel in which every
 * wavefront of the chip issues bf16 32x32x16 MFMAs back to back from registers, `iters` times 32
 * of them, 8 wavefronts per CU. The rate it reaches is the practical MFMA ceiling FOR THE GIVEN
 * OPERAND VALUES: the chip lowers its clock under the power that toggling operand bits costs.
 *   data    device, at least 64 KiB, 16-byte aligned: the bf16 values used as operands
 *   sink    device, at least 4 bytes (written practically never; keeps the loop alive)
 *   flop    host, out: floating-point operations the launch executes (time it with events)
 * Returns MLT_OK, MLT_ERR_INVALID_ARG (null pointer, iters outside 1 .. 2^20) or a launch/device
 * error.
 */
int mlt_probe_mfma(int iters, const void* data, void* sink, double* flop, void* stream);

/*
 * The same diagnostic on 16x16x32 MFMAs (64 per iteration and wavefront, the same flop count):
 * the shape the big-tile GEMM uses. On N(0,1) operands the chip sustains a higher rate of these
 * than of 32x32x16 MFMAs (it is power-limited, and this shape reads and writes half as many
 * accumulator registers per flop). Arguments and return values as for mlt_probe_mfma.
 */
int mlt_probe_mfma16(int iters, const void* data, void* sink, double* flop, void* stream);

/*
 * Diagnostic for benchmarks (not part of the paper's method): enqueues one kernel that reads
 * `bytes` bytes at `data` once with 16-byte loads from every CU and writes nothing. On a buffer
 * much larger than the caches its duration gives the practical HBM read rate, the ceiling for
 * the memory-bound kernels here (paged-attention decode, skinny GEMM).
 *   data    device, 16-byte aligned, `bytes` bytes (a positive multiple of 16); only read
 *   sink    device, at least 4 bytes (never written in practice; keeps the loads alive)
 * Returns MLT_OK, MLT_ERR_INVALID_ARG (null pointer, bad size or alignment) or a launch/device
 * error.
 */
int mlt_probe_hbm_read(const void* data, int64_t bytes, void* sink, void* stream);

/*
 * Per-kernel timing hook for benchmarks: when `start_event`/`stop_event` (hipEvent_t as void*,
 * may be NULL) are set, the next launches made by this thread record them on the launch stream
 * immediately before the first and after the last kernel of one entry-point call. Pass NULLs to
 * switch it off. Host-side state only; thread-local.
 */
void mlt_set_timing_events(void* start_event, void* stop_event);

/*
 * Name of the kernel variant the last successful call on this thread selected (static string,
 * e.g. "gemm_bf16_nn_256x256x64"); "" before any call. For logs and profiles.
 */
const char* mlt_last_kernel(void);

/*
 * Host-only query of the tiling a call would use, mirroring the paper's layout encoding
 * (Section 2.1: sizePerWarp and warpsPerCTA of the root operation). Fills
 *   out[0..1] workgroup tile (rows, cols), out[2..3] wavefronts per workgroup (rows, cols),
 *   out[4..5] sub-tile per wavefront, out[6..8] MFMA tile (m, n, k), out[9] K step (GEMM) or key
 *   tile (attention).
 * `op` 0 = GEMM (dims = M, N, K, transB), 1 = attention (dims = Sq, Sk, D, causal).
 * Returns MLT_OK or an error as the compute call would.
 */
int mlt_query_tiling(int op, const int64_t dims[4], int dtype, int32_t out[10]);

/*
 * Overrides the automatic kernel choice of the GEMM entry points and of mlt_mha_fwd for the whole
 * process, for tuning and for tests that have to reach every kernel. A NULL argument leaves that
 * choice as it is; "" or "auto" restores the automatic choice. A forced kernel that cannot take a
 * problem (alignment, shape) falls back to one that can, as the automatic choice would.
 *   gemm_variant  "general", "256", "256w8", "256pp16", "128pp16", "128pp16k128", "256w4", "256w8x1",
 *                 "256w1x8", "128w8", "64x128", "64", "128k2", "64x128k2", "64k4", "skinny", "skinnydma"
 *   mha_variant   "pp32", "pp16", "ps"
 * The initial values come from the environment variables MLT_GEMM_VARIANT and MLT_MHA_VARIANT,
 * which are read once, at the first call that needs them. Not synchronised with compute calls
 * running on other threads. Returns MLT_OK, or MLT_ERR_INVALID_ARG for an unknown name (nothing
 * changes then).
 */
int mlt_diag_force_variant(const char* gemm_variant, const char* mha_variant);

/*
 * Number of parts the GEMM entry points split K into across workgroups (the small-tile kernels;
 * partial products through an fp32 scratch, added in a fixed order by a second kernel): 0 = the
 * cost model's choice (the default), 1 = never split, 2 / 4 / 8 = that many parts wherever every
 * part keeps at least 8 K steps of 64. Process-wide, like mlt_diag_force_variant. Returns MLT_OK
 * or MLT_ERR_INVALID_ARG.
 */
int mlt_diag_force_k_parts(int parts);

/*
 * Number of key ranges per (sequence, head) that mlt_paged_attn_decode spreads over workgroups:
 * 0 = the library's choice (the default: 1 while sequences x heads alone fill the chip, more
 * otherwise), 1..64 = that many (ranges beyond the end of a short sequence stay empty).
 * Process-wide. Returns MLT_OK or MLT_ERR_INVALID_ARG.
 */
int mlt_diag_force_key_split(int ranges);

/*
 * Number of workgroups the persistent attention kernel launches (0: one per CU, the default);
 * small values make every workgroup walk through many items even on a small problem. Initial
 * value from MLT_MHA_PS_GRID, read once. Returns MLT_OK or MLT_ERR_INVALID_ARG (negative or
 * >= 2^20).
 */
int mlt_diag_set_persistent_grid(int workgroups);

#ifdef __cplusplus
}
#endif
#endif /* MLT_DIAG_H_ */
