/*
 * CPU oracle for the two dense tile kernels of arXiv 2503.14985 ("ML-Triton"):
 *   - GEMM, Section 2 (the C = A*B example, 16-bit inputs with 32-bit accumulate in Listing 1)
 *   - attention forward, Section 2.5, Algorithm 1 (FlashAttention-2 forward)
 *   - paged attention for decoding, Section 3.2 (one query per sequence, keys and values in
 *     fixed-size blocks of a cache that a per-sequence block table maps to logical positions)
 *
 * THIS IS TEST INFRASTRUCTURE, not a product path. Only the tests, the smoke check and the
 * bench's cpu_baseline leg may call it. It shares no code with the GPU library.
 *
 * Both results have a plain mathematical definition, so the oracle is that definition written
 * out in fp64 with straight loops: no tiling, no online softmax, no reordering. The only
 * parallelism is an OpenMP split of the outermost independent loop (rows / samples), which
 * changes no arithmetic.
 *
 * Inputs are the raw 16-bit patterns (bf16 or IEEE fp16) that the GPU sees. Each is widened
 * exactly to double by the bit-level converters below.
 *
 * dtype: 0 = bf16, 1 = fp16.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- 16-bit <-> wide converters */

/* bf16 is the upper half of an IEEE binary32: widen by appending 16 zero bits. */
double oracle_bf16_to_f64(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_f16_to_f64(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int frac = h & 0x3ff;
  double v;
  if (e == 0) {
    v = ldexp((double)frac, -24); /* zero and subnormals: frac * 2^-10 * 2^-14 */
  } else if (e == 31) {
    v = frac ? NAN : INFINITY;
  } else {
    v = ldexp(1.0 + (double)frac / 1024.0, e - 15);
  }
  return sign ? -v : v;
}

static inline double widen(uint16_t h, int dtype) {
  return dtype == 0 ? oracle_bf16_to_f64(h) : oracle_f16_to_f64(h);
}

/*
 * Round a double to the nearest value of the 16-bit format, ties to even, and return that value
 * as a double (used by tests to separate output-rounding error from arithmetic error).
 * Works on the exact binary expansion: scale so that one unit in the last place is 1.0, round
 * with the ties-to-even rule, scale back.
 */
double oracle_round_to_dtype(double x, int dtype) {
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  const int mant_bits = dtype == 0 ? 7 : 10;   /* explicit fraction bits */
  const int min_exp = dtype == 0 ? -126 : -14; /* exponent of the smallest normal */
  const int max_exp = dtype == 0 ? 127 : 15;
  int e;
  double a = fabs(x);
  frexp(a, &e);     /* a = f * 2^e, f in [0.5, 1)  =>  exponent of leading bit is e-1 */
  int lead = e - 1;
  if (lead < min_exp) lead = min_exp;          /* subnormal range: fixed ulp */
  int ulp_exp = lead - mant_bits;
  double scaled = ldexp(a, -ulp_exp);          /* exact: power-of-two scaling */
  double fl = floor(scaled);
  double rem = scaled - fl;
  double r;
  if (rem > 0.5) r = fl + 1.0;
  else if (rem < 0.5) r = fl;
  else r = (fmod(fl, 2.0) == 0.0) ? fl : fl + 1.0;
  double out = ldexp(r, ulp_exp);
  double max_finite = ldexp(2.0 - ldexp(1.0, -mant_bits), max_exp);
  if (out > max_finite) out = INFINITY;
  return x < 0 ? -out : out;
}

/* Widen n patterns to doubles in one call. */
void oracle_widen_array(const uint16_t* bits, int64_t n, double* out, int dtype) {
  for (int64_t i = 0; i < n; ++i) out[i] = widen(bits[i], dtype);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static void set_threads(int nthreads) {
#ifdef _OPENMP
  if (nthreads > 0) omp_set_num_threads(nthreads);
#else
  (void)nthreads;
#endif
}

/* ------------------------------------------------------------------------------------ GEMM */

/* Element (k, j) of the K x N matrix B. transB = 1 means the buffer holds the N x K row-major
 * transpose (i.e. B in column-major order), with ldb the stride between its rows. */
static inline double b_at(const uint16_t* B, int64_t ldb, int transB, int64_t k, int64_t j,
                          int dtype) {
  return widen(transB ? B[j * ldb + k] : B[k * ldb + j], dtype);
}

/*
 * One output element of C = A*B by its definition (Section 2: A is m x k, B is k x n):
 *   c = sum_k a[i][k] * b[k][j],      t = sum_k |a[i][k]| * |b[k][j]|
 * t is the magnitude sum that the parity tolerance is scaled by.
 */
static void gemm_element(int64_t K, const uint16_t* A, int64_t lda, const uint16_t* B,
                         int64_t ldb, int transB, int dtype, int64_t i, int64_t j, double* c,
                         double* t) {
  double acc = 0.0, mag = 0.0;
  for (int64_t k = 0; k < K; ++k) {
    double a = widen(A[i * lda + k], dtype);
    double b = b_at(B, ldb, transB, k, j, dtype);
    acc += a * b;
    mag += fabs(a) * fabs(b);
  }
  *c = acc;
  *t = mag;
}

/* Full product. C_ref and T are M x N row-major doubles (leading dimension N); T may be NULL. */
int oracle_gemm(int64_t M, int64_t N, int64_t K, const uint16_t* A, int64_t lda,
                const uint16_t* B, int64_t ldb, int transB, double* C_ref, double* T, int dtype,
                int nthreads) {
  if (M < 0 || N < 0 || K < 0 || (dtype != 0 && dtype != 1)) return -1;
  set_threads(nthreads);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      double c, t;
      gemm_element(K, A, lda, B, ldb, transB, dtype, i, j, &c, &t);
      C_ref[i * N + j] = c;
      if (T) T[i * N + j] = t;
    }
  }
  return 0;
}

/* The same definition evaluated only at the listed (rows[s], cols[s]) positions. */
int oracle_gemm_sampled(int64_t M, int64_t N, int64_t K, const uint16_t* A, int64_t lda,
                        const uint16_t* B, int64_t ldb, int transB, int64_t nsamples,
                        const int64_t* rows, const int64_t* cols, double* C_ref, double* T,
                        int dtype, int nthreads) {
  if (M < 0 || N < 0 || K < 0 || nsamples < 0 || (dtype != 0 && dtype != 1)) return -1;
  for (int64_t s = 0; s < nsamples; ++s)
    if (rows[s] < 0 || rows[s] >= M || cols[s] < 0 || cols[s] >= N) return -1;
  set_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t s = 0; s < nsamples; ++s) {
    double c, t;
    gemm_element(K, A, lda, B, ldb, transB, dtype, rows[s], cols[s], &c, &t);
    C_ref[s] = c;
    if (T) T[s] = t;
  }
  return 0;
}

/*
 * Epilogue of the fused GEMM (the post-operation fusion remark of Section 3.1): applied in place
 * to exact products x = (A*B)[i][j] held in fp64, row-major with row stride ldx,
 *   y = act(x + bias[j]),   bias one value per COLUMN in the 16-bit input type (or none),
 *   act 0: identity, 1: ReLU max(y, 0), 2: GELU in its exact form y * Phi(y) with the standard
 *   normal distribution function Phi(y) = (1 + erf(y / sqrt 2)) / 2.
 * mag, if given, holds the magnitude sums |A||B| and receives + |bias[j]| (the scale the parity
 * tolerance is relative to).
 */
int oracle_gemm_epilogue(int64_t M, int64_t N, double* X, int64_t ldx, double* mag,
                         const uint16_t* bias, int act, int dtype) {
  if (M < 0 || N < 0 || act < 0 || act > 2 || (dtype != 0 && dtype != 1)) return -1;
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      double y = X[i * ldx + j];
      if (bias) {
        const double bj = widen(bias[j], dtype);
        y += bj;
        if (mag) mag[i * ldx + j] += fabs(bj);
      }
      if (act == 1) y = y > 0.0 ? y : 0.0;
      if (act == 2) y = 0.5 * y * (1.0 + erf(y / sqrt(2.0)));
      X[i * ldx + j] = y;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------------- attention */

/*
 * One output row of attention for head (b, h), query row i (Algorithm 1 computes exactly
 * softmax(scale * Q K^T [+ causal mask]) V, blockwise; here it is the plain row formula):
 *   s_j = scale * sum_d q[i][d] k[j][d]      for every visible key j
 *   w_j = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *   o[:] = sum_j w_j v[j][:]
 * Visible keys: all j in [0, Sk) without the mask; j <= i with the causal mask (lower triangle
 * including the diagonal, aligned at the top-left corner, so key 0 is always visible).
 * Masked keys are left out of every sum rather than given a large negative score.
 * Tensors are contiguous [B, H, S, D]. `w` (length Sk, may be NULL) receives the weights, with
 * zeros at masked positions; `scratch` must hold Sk doubles.
 */
static void mha_row(int64_t H, int64_t Sq, int64_t Sk, int64_t D, const uint16_t* Q,
                    const uint16_t* Kt, const uint16_t* V, double scale, int causal, int dtype,
                    int64_t b, int64_t h, int64_t i, double* o, double* w, double* scratch) {
  const uint16_t* q = Q + ((b * H + h) * Sq + i) * D;
  const uint16_t* kbase = Kt + (b * H + h) * Sk * D;
  const uint16_t* vbase = V + (b * H + h) * Sk * D;
  int64_t nvis = causal ? (i + 1 < Sk ? i + 1 : Sk) : Sk;
  double* s = scratch;
  double m = -INFINITY;
  for (int64_t j = 0; j < nvis; ++j) {
    double dot = 0.0;
    for (int64_t d = 0; d < D; ++d) dot += widen(q[d], dtype) * widen(kbase[j * D + d], dtype);
    s[j] = scale * dot;
    if (s[j] > m) m = s[j];
  }
  double l = 0.0;
  for (int64_t j = 0; j < nvis; ++j) {
    s[j] = exp(s[j] - m);
    l += s[j];
  }
  for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
  for (int64_t j = 0; j < nvis; ++j) {
    double wj = s[j] / l;
    if (w) w[j] = wj;
    for (int64_t d = 0; d < D; ++d) o[d] += wj * widen(vbase[j * D + d], dtype);
  }
  if (w)
    for (int64_t j = nvis; j < Sk; ++j) w[j] = 0.0;
}

/* All rows. O_ref is [B, H, Sq, D] doubles. */
int oracle_mha_fwd(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const uint16_t* Q,
                   const uint16_t* K, const uint16_t* V, double* O_ref, double scale, int causal,
                   int dtype, int nthreads) {
  if (B < 0 || H < 0 || Sq < 0 || Sk <= 0 || D <= 0 || (dtype != 0 && dtype != 1)) return -1;
  set_threads(nthreads);
  int64_t nrows = B * H * Sq;
  int fail = 0;
#pragma omp parallel
  {
    double* scratch = (double*)__builtin_malloc(sizeof(double) * (size_t)Sk);
    if (!scratch) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 16)
    for (int64_t r = 0; r < nrows; ++r) {
      if (!scratch) continue;
      int64_t i = r % Sq, bh = r / Sq;
      mha_row(H, Sq, Sk, D, Q, K, V, scale, causal, dtype, bh / H, bh % H, i, O_ref + r * D,
              (double*)0, scratch);
    }
    __builtin_free(scratch);
  }
  return fail ? -2 : 0;
}

/* Only the listed rows: row r is (bs[r], hs[r], is[r]); O_ref is [nrows, D]; W (may be NULL) is
 * [nrows, Sk] and receives the softmax weights of each row. */
int oracle_mha_fwd_rows(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D,
                        const uint16_t* Q, const uint16_t* K, const uint16_t* V, int64_t nrows,
                        const int64_t* bs, const int64_t* hs, const int64_t* is, double* O_ref,
                        double* W, double scale, int causal, int dtype, int nthreads) {
  if (B < 0 || H < 0 || Sq < 0 || Sk <= 0 || D <= 0 || nrows < 0 || (dtype != 0 && dtype != 1))
    return -1;
  for (int64_t r = 0; r < nrows; ++r)
    if (bs[r] < 0 || bs[r] >= B || hs[r] < 0 || hs[r] >= H || is[r] < 0 || is[r] >= Sq) return -1;
  set_threads(nthreads);
  int fail = 0;
#pragma omp parallel
  {
    double* scratch = (double*)__builtin_malloc(sizeof(double) * (size_t)Sk);
    if (!scratch) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < nrows; ++r) {
      if (!scratch) continue;
      mha_row(H, Sq, Sk, D, Q, K, V, scale, causal, dtype, bs[r], hs[r], is[r], O_ref + r * D,
              W ? W + r * Sk : (double*)0, scratch);
    }
    __builtin_free(scratch);
  }
  return fail ? -2 : 0;
}

/* ------------------------------------------------------------------ paged attention, decoding */

/*
 * Section 3.2 of the paper: attention of ONE query per (sequence b, head h) over that sequence's
 * cached keys and values, o = sum_j softmax_j(scale * q.k_j) v_j, j = 0 .. seq_len[b]-1. The
 * paper fixes no storage layout; the one used here (and by the GPU library) is
 *   Q, O          [B, H, D]
 *   Kc, Vc        [num_blocks, H, block_size, D]   (the cache: physical blocks)
 *   block_table   [B, max_blocks] int32: physical block of logical block i of sequence b
 *   seq_lens      [B] int32, 1 <= seq_len[b] <= max_blocks * block_size
 * Logical key position p of sequence b is slot p % block_size of physical block
 * block_table[b][p / block_size]. Table entries and cache slots beyond seq_len are never read.
 * The definition is written out directly: gather, scores, maximum, exponentials, weighted sum,
 * all in double; the split over wavefronts and the cross-wavefront reduction that the paper
 * describes are the GPU method, not part of the definition.
 * Returns 0, -1 for bad arguments (including a table entry outside [0, num_blocks)), -2 when out
 * of memory. W (may be NULL) is [B, H, max_blocks * block_size] and receives the weights (zero
 * beyond seq_len).
 */
int oracle_paged_attn_decode(int64_t B, int64_t H, int64_t D, int64_t block_size,
                             int64_t max_blocks, int64_t num_blocks, const uint16_t* Q,
                             const uint16_t* Kc, const uint16_t* Vc, const int32_t* block_table,
                             const int32_t* seq_lens, double* O_ref, double* W, double scale,
                             int dtype, int nthreads) {
  if (B < 0 || H < 0 || D <= 0 || block_size <= 0 || max_blocks <= 0 || num_blocks <= 0 ||
      (dtype != 0 && dtype != 1))
    return -1;
  for (int64_t b = 0; b < B; ++b) {
    int64_t len = seq_lens[b];
    if (len < 1 || len > max_blocks * block_size) return -1;
    for (int64_t i = 0; i * block_size < len; ++i) {
      int64_t pb = block_table[b * max_blocks + i];
      if (pb < 0 || pb >= num_blocks) return -1;
    }
  }
  set_threads(nthreads);
  int fail = 0;
  const int64_t cap = max_blocks * block_size;
#pragma omp parallel
  {
    double* s = (double*)__builtin_malloc(sizeof(double) * (size_t)cap);
    if (!s) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 4)
    for (int64_t r = 0; r < B * H; ++r) {
      if (!s) continue;
      const int64_t b = r / H, h = r % H, len = seq_lens[b];
      const uint16_t* q = Q + r * D;
      double m = -INFINITY;
      for (int64_t p = 0; p < len; ++p) {
        const int64_t pb = block_table[b * max_blocks + p / block_size];
        const uint16_t* k = Kc + ((pb * H + h) * block_size + p % block_size) * D;
        double dot = 0.0;
        for (int64_t d = 0; d < D; ++d) dot += widen(q[d], dtype) * widen(k[d], dtype);
        s[p] = scale * dot;
        if (s[p] > m) m = s[p];
      }
      double l = 0.0;
      for (int64_t p = 0; p < len; ++p) {
        s[p] = exp(s[p] - m);
        l += s[p];
      }
      double* o = O_ref + r * D;
      for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t p = 0; p < len; ++p) {
        const int64_t pb = block_table[b * max_blocks + p / block_size];
        const uint16_t* v = Vc + ((pb * H + h) * block_size + p % block_size) * D;
        const double wp = s[p] / l;
        if (W) W[r * cap + p] = wp;
        for (int64_t d = 0; d < D; ++d) o[d] += wp * widen(v[d], dtype);
      }
      if (W)
        for (int64_t p = len; p < cap; ++p) W[r * cap + p] = 0.0;
    }
    __builtin_free(s);
  }
  return fail ? -2 : 0;
}
