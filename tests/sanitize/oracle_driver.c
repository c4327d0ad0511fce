/* Runs every entry point of the fp64 oracle (oracle/oracle.c, compiled into this program with
 * -fsanitize=address,undefined) on small ragged problems whose buffers are exactly as large as the
 * documented layouts say, so that an access outside them or an undefined operation ends the
 * program with a sanitizer report. Prints "ok" and exits 0 otherwise. Test infrastructure. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double oracle_bf16_to_f64(uint16_t h);
double oracle_f16_to_f64(uint16_t h);
double oracle_round_to_dtype(double x, int dtype);
void oracle_widen_array(const uint16_t* bits, int64_t n, double* out, int dtype);
int oracle_gemm(int64_t M, int64_t N, int64_t K, const uint16_t* A, int64_t lda, const uint16_t* B,
                int64_t ldb, int transB, double* C_ref, double* T, int dtype, int nthreads);
int oracle_gemm_sampled(int64_t M, int64_t N, int64_t K, const uint16_t* A, int64_t lda,
                        const uint16_t* B, int64_t ldb, int transB, int64_t nsamples,
                        const int64_t* rows, const int64_t* cols, double* C_ref, double* T,
                        int dtype, int nthreads);
int oracle_gemm_epilogue(int64_t M, int64_t N, double* X, int64_t ldx, double* mag,
                         const uint16_t* bias, int act, int dtype);
int oracle_mha_fwd(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const uint16_t* Q,
                   const uint16_t* K, const uint16_t* V, double* O_ref, double scale, int causal,
                   int dtype, int nthreads);
int oracle_mha_fwd_rows(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const uint16_t* Q,
                        const uint16_t* K, const uint16_t* V, int64_t nrows, const int64_t* bs,
                        const int64_t* hs, const int64_t* is, double* O_ref, double* W, double scale,
                        int causal, int dtype, int nthreads);
int oracle_paged_attn_decode(int64_t B, int64_t H, int64_t D, int64_t block_size,
                             int64_t max_blocks, int64_t num_blocks, const uint16_t* Q,
                             const uint16_t* Kc, const uint16_t* Vc, const int32_t* block_table,
                             const int32_t* seq_lens, double* O_ref, double* W, double scale,
                             int dtype, int nthreads);

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state;
}
/* a finite 16-bit pattern of modest magnitude (exponent field kept in the middle of its range) */
static uint16_t small_value(int dtype) {
  const uint32_t r = next_u32();
  if (dtype == 0) return (uint16_t)(((r >> 16) & 0x8000u) | (0x3e00u + ((r >> 8) & 0x1ffu)));
  return (uint16_t)(((r >> 16) & 0x8000u) | (0x3000u + ((r >> 8) & 0xfffu)));
}
static uint16_t* values(int64_t n, int dtype) {
  uint16_t* p = (uint16_t*)malloc((size_t)(n > 0 ? n : 1) * sizeof(uint16_t));
  for (int64_t i = 0; i < n; ++i) p[i] = small_value(dtype);
  return p;
}
#define CHECK(x) do { if (!(x)) { printf("failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void) {
  for (int dtype = 0; dtype < 2; ++dtype) {
    /* converters over every pattern */
    for (uint32_t h = 0; h < 65536u; ++h) {
      const double x = dtype == 0 ? oracle_bf16_to_f64((uint16_t)h) : oracle_f16_to_f64((uint16_t)h);
      if (x == x) (void)oracle_round_to_dtype(x * 1.0009765625, dtype);
    }
    (void)oracle_round_to_dtype(1e300, dtype);
    (void)oracle_round_to_dtype(-1e-300, dtype);
    /* GEMM, both storage orders of B, padded leading dimensions, sizes with no factor of 2 */
    for (int transB = 0; transB < 2; ++transB) {
      const int64_t M = 7, N = 5, K = 11, lda = K + 3, ldb = (transB ? K : N) + 2;
      uint16_t* A = values((M - 1) * lda + K, dtype);
      uint16_t* B = values(transB ? (N - 1) * ldb + K : (K - 1) * ldb + N, dtype);
      double* C = (double*)malloc(M * N * sizeof(double));
      double* T = (double*)malloc(M * N * sizeof(double));
      CHECK(oracle_gemm(M, N, K, A, lda, B, ldb, transB, C, T, dtype, 2) == 0);
      int64_t rows[4] = {0, 6, 3, 6}, cols[4] = {4, 0, 2, 4};
      double cs[4], ts[4];
      CHECK(oracle_gemm_sampled(M, N, K, A, lda, B, ldb, transB, 4, rows, cols, cs, ts, dtype, 2) == 0);
      CHECK(cs[1] == C[6 * N + 0] && cs[3] == C[6 * N + 4]);
      uint16_t* bias = values(N, dtype);
      for (int act = 0; act < 3; ++act) CHECK(oracle_gemm_epilogue(M, N, C, N, T, bias, act, dtype) == 0);
      CHECK(oracle_gemm(M, N, 0, A, lda, B, ldb, transB, C, T, dtype, 1) == 0);      /* K = 0 */
      CHECK(oracle_gemm(0, N, K, A, lda, B, ldb, transB, C, T, dtype, 1) == 0);      /* no rows */
      CHECK(oracle_gemm(-1, N, K, A, lda, B, ldb, transB, C, T, dtype, 1) != 0);
      free(A); free(B); free(C); free(T); free(bias);
    }
    /* attention, rectangular, with and without the mask; then selected rows with weights */
    for (int causal = 0; causal < 2; ++causal) {
      const int64_t B = 2, H = 3, Sq = 5, Sk = 9, D = 8;
      uint16_t* Q = values(B * H * Sq * D, dtype);
      uint16_t* K = values(B * H * Sk * D, dtype);
      uint16_t* V = values(B * H * Sk * D, dtype);
      double* O = (double*)malloc(B * H * Sq * D * sizeof(double));
      CHECK(oracle_mha_fwd(B, H, Sq, Sk, D, Q, K, V, O, 0.35, causal, dtype, 2) == 0);
      int64_t bs[3] = {1, 0, 1}, hs[3] = {2, 0, 1}, is[3] = {4, 0, 2};
      double Or[3 * 8], W[3 * 9];
      CHECK(oracle_mha_fwd_rows(B, H, Sq, Sk, D, Q, K, V, 3, bs, hs, is, Or, W, 0.35, causal, dtype, 2) == 0);
      CHECK(Or[0] == O[((1 * H + 2) * Sq + 4) * D]);
      CHECK(oracle_mha_fwd_rows(B, H, Sq, Sk, D, Q, K, V, 3, bs, hs, is, Or, NULL, -0.2, causal, dtype, 1) == 0);
      CHECK(oracle_mha_fwd(B, H, Sq, 0, D, Q, K, V, O, 0.35, causal, dtype, 1) != 0);   /* no keys */
      free(Q); free(K); free(V); free(O);
    }
    /* paged decode: shuffled blocks, lengths from one key to the whole table */
    {
      const int64_t B = 3, H = 2, D = 8, bs = 4, max_blocks = 3, num_blocks = 9;
      uint16_t* Q = values(B * H * D, dtype);
      uint16_t* Kc = values(num_blocks * H * bs * D, dtype);
      uint16_t* Vc = values(num_blocks * H * bs * D, dtype);
      int32_t table[9] = {8, 0, 4, 2, 7, 1, 3, 5, 6};
      int32_t lens[3] = {1, 12, 7};
      double O[3 * 2 * 8], W[3 * 2 * 12];
      CHECK(oracle_paged_attn_decode(B, H, D, bs, max_blocks, num_blocks, Q, Kc, Vc, table, lens, O, W, 0.5, dtype, 2) == 0);
      CHECK(oracle_paged_attn_decode(B, H, D, bs, max_blocks, num_blocks, Q, Kc, Vc, table, lens, O, NULL, 0.5, dtype, 1) == 0);
      free(Q); free(Kc); free(Vc);
    }
  }
  printf("ok\n");
  return 0;
}
