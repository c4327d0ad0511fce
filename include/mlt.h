/*
 * mlt — tile-based dense kernels for AMD MI355X (gfx950, CDNA4, wave64), C ABI.
 *
 * The two operations are the dense workloads that arXiv 2503.14985 ("ML-Triton") lowers
 * workgroup -> warp -> intrinsic: a 16-bit GEMM with 32-bit accumulation (Section 2, Listing 1)
 * and a FlashAttention-2-style attention forward (Section 2.5, Algorithm 1). Here both are
 * hand-written HIP kernels; the workgroup tile -> per-wavefront sub-tile -> MFMA tile split is
 * fixed at compile time per kernel variant.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers to memory the caller owns. The library never frees
 *     or keeps them. Inputs and outputs must not overlap.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Work is enqueued
 *     asynchronously on it; no entry point synchronises the device.
 *   - `dtype` selects the 16-bit element type of every input and output tensor:
 *     MLT_BF16 (bfloat16) or MLT_FP16 (IEEE binary16). Accumulation is fp32; outputs are
 *     rounded to `dtype` with round-to-nearest-even.
 *   - Return value: MLT_OK or a negative mlt_status. No C++ exception crosses the boundary and
 *     nothing aborts. On an error nothing has been enqueued.
 *   - Device memory of the library's own: the GEMM entry points (few tiles against a long K) and
 *     mlt_paged_attn_decode (few sequences x heads) may spread one result over several workgroups
 *     and then keep fp32 partial results in a scratch buffer, one per (device, stream), allocated
 *     with hipMalloc at the first call that needs it, grown by doubling from 4 MiB (16 MiB covers
 *     every split the library chooses by itself) and kept until the process ends. Calls on one
 *     stream are ordered by the stream; calls on different streams use different buffers. If the
 *     allocation fails, or the stream is recording into a graph and has no buffer yet, the call
 *     runs without the split (same result up to summation order). mlt_gemm_noalloc never
 *     allocates.
 */
#ifndef MLT_H_
#define MLT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MLT_BF16 = 0, MLT_FP16 = 1 } mlt_dtype;

typedef enum {
  MLT_OK = 0,
  MLT_ERR_INVALID_ARG = -1, /* null pointer, negative size, leading dimension too small, bad dtype */
  MLT_ERR_UNSUPPORTED = -2, /* valid request with no kernel (e.g. head dimension not 64 or 128) */
  MLT_ERR_LAUNCH = -3,      /* the HIP runtime rejected the kernel launch */
  MLT_ERR_DEVICE = -4,      /* no usable gfx950 device is current */
  MLT_ERR_SCRATCH = -5      /* mlt_gemm_noalloc: the call needs more than the fixed scratch array holds */
} mlt_status;

/*
 * GEMM, Section 2 of the paper (A is m x k, B is k x n, C is m x n; 16-bit inputs, fp32
 * accumulate as in Listing 1). Computes C = A * B, overwriting C (no accumulation into the
 * previous contents), output rounded to `dtype`.
 *
 *   A      device, M x K row-major, row stride lda >= K elements
 *   B      device; transB == 0: K x N row-major, row stride ldb >= N
 *                  transB != 0: the N x K row-major array holding B transposed (B in
 *                               column-major order), row stride ldb >= K
 *   C      device, M x N row-major, row stride ldc >= N; written, never read
 *
 * M, N or K may be 0: M == 0 or N == 0 is a no-op, K == 0 stores zeros. Any positive shape and
 * any leading dimensions/alignments are accepted; shapes and pointers that allow 16-byte vector
 * access (K, N, lda, ldb multiples of 8 and 16-byte aligned bases) take the fast kernels, others
 * a slower general kernel with identical results up to summation order.
 */
int mlt_gemm(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
             int64_t ldb, int transB, void* C, int64_t ldc, int dtype, void* stream);

/*
 * mlt_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. Same arguments, same kernels and the same
 * result, bit for bit, as mlt_gemm. Where mlt_gemm splits K across workgroups (few tiles against
 * a long K) and keeps the fp32 partial products in a scratch buffer it allocates, this entry point
 * keeps them in a fixed array of 32 MiB in device memory that is part of the library (one copy
 * per GPU the library runs on, held until the process ends). It calls no hipMalloc, hipFree or
 * other allocating routine. The library's own choice of a split never needs more than 16 MiB;
 * a split forced through mlt_diag_force_k_parts that needs more than 32 MiB (parts * M * N * 4
 * bytes) is refused with MLT_ERR_SCRATCH and nothing is enqueued. All calls on one GPU share that
 * GPU's array: two calls of this entry point that may run at the same time on one GPU (different
 * streams) race; calls on one stream, and calls on different GPUs, do not.
 */
int mlt_gemm_noalloc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                     int64_t ldb, int transB, void* C, int64_t ldc, int dtype, void* stream);

/*
 * The paper's own form of the GEMM (Section 2, Listing 1): C += A * B with C in fp32, i.e. the
 * fp32 accumulator is added to what C already holds and nothing is rounded to 16 bit.
 * A, B, transB, dtype as for mlt_gemm; C is device, M x N row-major fp32, row stride ldc >= N
 * (in fp32 elements), 4-byte aligned, read and written. M, N or K equal to 0 is a no-op. The
 * read-modify-write of C is not atomic: do not run two calls on the same C concurrently.
 */
int mlt_gemm_acc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                 int64_t ldb, int transB, float* C, int64_t ldc, int dtype, void* stream);

/*
 * mlt_gemm with the paper's `tiling` hint (Section 3.1, "Compiler Hint"): how the wavefronts of a
 * workgroup divide its 256 x 256 output tile. All settings compute the same C (up to summation
 * order) and obey the same tolerances; what changes is the kernel.
 *   tiling 0  the library's choice (the same as mlt_gemm)
 *          1  horizontal: evenly along the rows only, 8 wavefronts x (32 x 256)
 *          2  vertical: evenly along the columns only, 8 wavefronts x (256 x 32)
 *          3  square: 2 x 2 wavefronts x (128 x 128)
 * The hint applies to operands that allow 16-byte vector access (see mlt_gemm); others take the
 * general kernel, K = 0 stores zeros, and the skinny kernels (M <= 32 with B stored N x K) and
 * the smaller workgroup tiles of small problems are chosen only for tiling 0. Returns as mlt_gemm; MLT_ERR_INVALID_ARG also for an unknown `tiling`.
 */
int mlt_gemm_tiled(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                   int64_t ldb, int transB, void* C, int64_t ldc, int dtype, int tiling,
                   void* stream);

/*
 * GEMM with a fused epilogue, C = act(A*B + bias): the post-operation fusion the paper expects to
 * fall out of its layout propagation from the root operation (Section 3.1, the remark on pre- and
 * post-operation fusion), here written into the kernels' epilogues. Arguments as for mlt_gemm,
 * plus
 *   bias   device, N elements of `dtype` added to every row of A*B in fp32 before the activation,
 *          or NULL for none; only read
 *   act    0 none, 1 ReLU max(x, 0), 2 GELU in its exact form x * Phi(x) = x/2 * (1 + erf(x/sqrt 2))
 * The fp32 accumulator plus bias goes through the activation in fp32 and is rounded once (RNE) to
 * the 16-bit C. K = 0 gives C = act(bias) (act(0) without a bias). Returns as mlt_gemm;
 * MLT_ERR_INVALID_ARG also for an unknown `act` or a misaligned bias.
 */
int mlt_gemm_bias_act(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                      int64_t ldb, int transB, const void* bias, int act, void* C, int64_t ldc,
                      int dtype, void* stream);

/*
 * Attention forward, Section 2.5 / Algorithm 1 of the paper, per batch b and head h:
 *   O = softmax(scale * Q K^T  [+ causal mask]) V
 * computed tile by tile with the online-softmax recurrence (running row maximum m and row sum
 * l in fp32, P rounded to `dtype` before the second product, one division by l at the end).
 *
 *   Q, O   device, contiguous [B, H, Sq, D], D innermost
 *   K, V   device, contiguous [B, H, Sk, D]
 *   causal != 0: key j is visible to query i iff j <= i (lower triangle including the
 *                diagonal, aligned at the top-left corner; key 0 is visible to every query).
 *
 * D must be 64 or 128 and one head's K must stay below 2 GiB (Sk * D * 2 < 2^31), else
 * MLT_ERR_UNSUPPORTED. B, H or Sq equal to 0 is a no-op. Sk must be >= 1 (a softmax over no keys
 * is undefined: MLT_ERR_INVALID_ARG). All four base pointers must be 16-byte aligned and scale
 * must be finite (MLT_ERR_INVALID_ARG otherwise).
 */
int mlt_mha_fwd(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const void* Q,
                const void* K, const void* V, void* O, float scale, int causal, int dtype,
                void* stream);

/*
 * Paged attention for decoding, Section 3.2 of the paper: ONE query per (sequence b, head h) over
 * the seq_lens[b] keys and values of that sequence, which live in fixed-size blocks of a cache:
 *   o = sum_j softmax_j(scale * q . k_j) v_j,   j = 0 .. seq_lens[b] - 1.
 * The keys are split over the wavefronts of a workgroup and the partial maxima, sums and outputs
 * are reduced through LDS (the paper's warp-level decomposition, Listing 6); with too few
 * sequences x heads to fill the chip the keys are split over several workgroups as well, whose
 * partial results a second kernel merges in a fixed order. Weights are rounded
 * to `dtype` before they multiply V (Listing 5). The paper fixes no storage layout; this one is
 *   Q, O          device, contiguous [B, H, D]
 *   Kc, Vc        device, contiguous [num_blocks, H, block_size, D]: the cache, physical blocks
 *   block_table   device, int32 [B, max_blocks]: physical block of logical block i of sequence b;
 *                 logical key p is slot p % block_size of block block_table[b][p / block_size]
 *   seq_lens      device, int32 [B], 1 <= seq_lens[b] <= max_blocks * block_size
 * Table entries past the last used block are never read; cache slots are read in units of 16
 * keys, so the slots from seq_lens[b] up to the next multiple of 16 inside the last used block are
 * read and ignored (their weights are forced to zero), nothing beyond them. The library cannot inspect
 * device data: an entry outside [0, num_blocks) or a length outside its range is CLAMPED into it
 * (wrong result for that sequence, no out-of-range access).
 * D must be 64 or 128, block_size a multiple of 16 up to 1024 (else MLT_ERR_UNSUPPORTED); Q, Kc
 * and Vc 16-byte aligned, scale finite (MLT_ERR_INVALID_ARG). B or H equal to 0 is a no-op.
 */
int mlt_paged_attn_decode(int64_t B, int64_t H, int64_t D, int64_t block_size, int64_t max_blocks,
                          int64_t num_blocks, const void* Q, const void* Kc, const void* Vc,
                          const int32_t* block_table, const int32_t* seq_lens, void* O,
                          float scale, int dtype, void* stream);

/* Static, human-readable text for a status code. */
const char* mlt_status_string(int status);

/* Static version string, "major.minor.patch". */
const char* mlt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MLT_H_ */
