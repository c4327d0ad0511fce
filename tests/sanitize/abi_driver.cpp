// Calls every compute entry point of the C ABI with arguments that the host-side checks must
// reject (or accept as a no-op) before anything touches a GPU, in a build whose host code (the
// argument validation and dispatch of csrc/mlt_api.hip) is compiled with
// -fsanitize=address,undefined. Needs no GPU. Prints "ok" and exits 0. Test infrastructure.
#include <stdint.h>
#include <stdio.h>

#include "../../include/mlt.h"
#include "../../include/mlt_diag.h"

#define CHECK(x) do { if (!(x)) { printf("failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main() {
  alignas(16) static uint16_t buf[64];      // stands in for device memory: never dereferenced
  void* p = buf;
  void* odd = reinterpret_cast<char*>(buf) + 2;
  // GEMM family: bad dtype, negative sizes, null operands, leading dimensions too small, no-ops
  CHECK(mlt_gemm(4, 4, 4, p, 4, p, 4, 0, p, 4, 7, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(-1, 4, 4, p, 4, p, 4, 0, p, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 4, 4, nullptr, 4, p, 4, 0, p, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 4, 4, p, 4, p, 4, 0, nullptr, 4, MLT_FP16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 4, 4, p, 3, p, 4, 0, p, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 6, 4, p, 4, p, 5, 0, p, 6, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 6, 4, p, 4, p, 3, 1, p, 6, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm(4, 6, 4, p, 4, p, 6, 0, p, 5, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm((int64_t)1 << 40, 4, 4, p, 4, p, 4, 0, p, 4, MLT_BF16, nullptr) == MLT_ERR_UNSUPPORTED);
  CHECK(mlt_gemm(0, 4, 4, nullptr, 4, nullptr, 4, 0, nullptr, 4, MLT_BF16, nullptr) == MLT_OK);
  CHECK(mlt_gemm(4, 0, 4, nullptr, 4, nullptr, 4, 1, nullptr, 0, MLT_FP16, nullptr) == MLT_OK);
  CHECK(mlt_gemm_noalloc(4, 4, 4, p, 3, p, 4, 0, p, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm_noalloc(0, 4, 4, nullptr, 4, nullptr, 4, 0, nullptr, 4, MLT_BF16, nullptr) == MLT_OK);
  CHECK(mlt_gemm_acc(4, 4, 4, p, 4, p, 4, 0, nullptr, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm_acc(0, 4, 4, nullptr, 4, nullptr, 4, 0, nullptr, 4, MLT_BF16, nullptr) == MLT_OK);
  CHECK(mlt_gemm_tiled(4, 4, 4, p, 4, p, 4, 0, p, 4, MLT_BF16, 99, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm_bias_act(4, 4, 4, p, 4, p, 4, 0, p, 9, p, 4, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_gemm_bias_act(0, 4, 4, nullptr, 4, nullptr, 4, 0, nullptr, 0, nullptr, 4, MLT_BF16, nullptr) == MLT_OK);
  // attention: head dimension, no keys, null and misaligned pointers, scale not finite, no-ops
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 96, p, p, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_UNSUPPORTED);
  CHECK(mlt_mha_fwd(1, 1, 8, 0, 64, p, p, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 64, nullptr, p, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 64, p, odd, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 64, p, p, p, p, 0.f / 0.f, 0, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 64, p, p, p, p, 1.f / 0.f, 1, MLT_FP16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(1, 1, 8, 8, 64, p, p, p, p, 1.f, 0, 5, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(-1, 1, 8, 8, 64, p, p, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_mha_fwd(0, 4, 8, 8, 64, nullptr, nullptr, nullptr, nullptr, 1.f, 0, MLT_BF16, nullptr) == MLT_OK);
  CHECK(mlt_mha_fwd(1, 1, 8, (int64_t)1 << 24, 128, p, p, p, p, 1.f, 0, MLT_BF16, nullptr) == MLT_ERR_UNSUPPORTED);
  // paged decode
  int32_t tbl[4] = {0, 0, 0, 0};
  CHECK(mlt_paged_attn_decode(1, 1, 96, 16, 1, 1, p, p, p, tbl, tbl, p, 1.f, MLT_BF16, nullptr) == MLT_ERR_UNSUPPORTED);
  CHECK(mlt_paged_attn_decode(1, 1, 64, 24, 1, 1, p, p, p, tbl, tbl, p, 1.f, MLT_BF16, nullptr) == MLT_ERR_UNSUPPORTED);
  CHECK(mlt_paged_attn_decode(1, 1, 64, 16, 0, 1, p, p, p, tbl, tbl, p, 1.f, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_paged_attn_decode(1, 1, 64, 16, 1, 1, p, p, p, nullptr, tbl, p, 1.f, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_paged_attn_decode(1, 1, 64, 16, 1, 1, p, odd, p, tbl, tbl, p, 1.f, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_paged_attn_decode(1, 1, 64, 16, 1, 1, p, p, p, tbl, tbl, p, 0.f / 0.f, MLT_BF16, nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_paged_attn_decode(0, 8, 64, 16, 1, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1.f, MLT_BF16, nullptr) == MLT_OK);
  // diagnostics: names, ranges, and the host-only tiling query
  CHECK(mlt_diag_force_variant("no such kernel", nullptr) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_diag_force_variant("auto", "auto") == MLT_OK);
  CHECK(mlt_diag_force_k_parts(3) == MLT_ERR_INVALID_ARG && mlt_diag_force_k_parts(0) == MLT_OK);
  CHECK(mlt_diag_force_key_split(65) == MLT_ERR_INVALID_ARG && mlt_diag_force_key_split(0) == MLT_OK);
  CHECK(mlt_diag_set_persistent_grid(-1) == MLT_ERR_INVALID_ARG && mlt_diag_set_persistent_grid(0) == MLT_OK);
  int64_t dims[4] = {8192, 8192, 8192, 0};
  int32_t out[10];
  CHECK(mlt_query_tiling(0, dims, MLT_BF16, out) == MLT_OK && out[0] == 256 && out[1] == 256);
  CHECK(mlt_query_tiling(0, nullptr, MLT_BF16, out) == MLT_ERR_INVALID_ARG);
  CHECK(mlt_query_tiling(5, dims, MLT_BF16, out) == MLT_ERR_INVALID_ARG);
  for (int code = 1; code >= -7; --code) CHECK(mlt_status_string(code) != nullptr);
  CHECK(mlt_version() != nullptr);
  printf("ok\n");
  return 0;
}
