// C ABI of the library: argument validation, variant selection, launch. No device work happens
// here besides enqueueing kernels on the caller's stream.
#include <limits.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/mlt_diag.h"
#include "mlt_common.h"
#include "mlt_internal.h"

using namespace mlt;

namespace {

thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
thread_local const char* g_last_kernel = "";
thread_local char g_name_buf[96];

// The selected kernel's name; a K split across workgroups shows as a suffix (_splitk2 / 4 / 8).
void note_gemm_kernel(const GemmPlan& p) {
  if (p.parts > 1) {
    snprintf(g_name_buf, sizeof(g_name_buf), "%s_splitk%d", p.name, p.parts);
    g_last_kernel = g_name_buf;
  } else {
    g_last_kernel = p.name;
  }
}

struct VariantName { const char* name; int id; };
const VariantName kGemmVariants[] = {
    {"general", GEMM_GENERAL}, {"256", GEMM_256}, {"256w8", GEMM_256_W8}, {"256pp16", GEMM_256_PP16}, {"128pp16", GEMM_128_PP16}, {"128pp16k128", GEMM_128_PP16_K128},
    {"256w4", GEMM_256_W4}, {"256w8x1", GEMM_256_W8X1}, {"256w1x8", GEMM_256_W1X8},
    {"128w8", GEMM_128_W8}, {"64x128", GEMM_64X128_W8}, {"64", GEMM_64_W4}, {"128k2", GEMM_128_K2},
    {"64x128k2", GEMM_64X128_K2}, {"64k4", GEMM_64_K4}, {"skinny", GEMM_SKINNY},
    {"skinnydma", GEMM_SKINNY_DMA}};
const VariantName kMhaVariants[] = {{"pp32", MHA_PP32}, {"pp16", MHA_PP16}, {"ps", MHA_PS}};

// name -> id; "" and "auto" mean the automatic choice; -2 for an unknown name
template <size_t N>
int lookup_variant(const VariantName (&table)[N], const char* name, int automatic) {
  if (!name || !*name || !strcmp(name, "auto")) return automatic;
  for (const auto& v : table)
    if (!strcmp(name, v.name)) return v.id;
  return -2;
}

Overrides overrides_from_env() {
  Overrides o;
  const int g = lookup_variant(kGemmVariants, getenv("MLT_GEMM_VARIANT"), GEMM_AUTO);
  if (g != -2) o.gemm = g;
  const int m = lookup_variant(kMhaVariants, getenv("MLT_MHA_VARIANT"), MHA_AUTO);
  if (m != -2) o.mha = m;
  if (const char* e = getenv("MLT_MHA_PS_GRID")) {
    const long v = strtol(e, nullptr, 10);
    if (v >= 1 && v < (1 << 20)) o.ps_grid = (int)v;
  }
  return o;
}

}  // namespace

namespace mlt {

// The environment is read once, when the first call needs the overrides.
Overrides& overrides() {
  static Overrides o = overrides_from_env();
  return o;
}

bool device_info(DeviceInfo& out) {
  static thread_local int cached_dev = -1;
  static thread_local DeviceInfo cached;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (dev != cached_dev) {
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, dev) != hipSuccess) { (void)hipGetLastError(); return false; }
    cached.gfx950 = strncmp(p.gcnArchName, "gfx950", 6) == 0;
    cached.ncu = p.multiProcessorCount;
    int xcds = 0;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess) (void)hipGetLastError();
    cached.nxcd = xcds > 0 ? xcds : 8;
    cached_dev = dev;
  }
  out = cached;
  return true;
}

int device_xcds() {
  DeviceInfo d;
  return device_info(d) && d.nxcd > 0 ? d.nxcd : 8;
}

}  // namespace mlt

namespace {

bool device_is_gfx950() {
  DeviceInfo d;
  return device_info(d) && d.gfx950;
}

int forced_gemm_variant() { return overrides().gemm; }

int check_gemm(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
               int64_t ldb, int transB, const void* C, int64_t ldc, int dtype) {
  if (dtype != MLT_BF16 && dtype != MLT_FP16) return MLT_ERR_INVALID_ARG;
  if (M < 0 || N < 0 || K < 0) return MLT_ERR_INVALID_ARG;
  if (M > INT_MAX || N > INT_MAX || K > INT_MAX) return MLT_ERR_UNSUPPORTED;
  if (M == 0 || N == 0) return MLT_OK;
  if (!C || ldc < N) return MLT_ERR_INVALID_ARG;
  if (K > 0) {
    if (!A || !B) return MLT_ERR_INVALID_ARG;
    if (lda < K) return MLT_ERR_INVALID_ARG;
    if (ldb < (transB ? K : N)) return MLT_ERR_INVALID_ARG;
  }
  return MLT_OK;
}

int check_mha(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const void* Q,
              const void* K, const void* V, const void* O, float scale, int dtype) {
  if (dtype != MLT_BF16 && dtype != MLT_FP16) return MLT_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || Sq < 0 || Sk < 0 || D <= 0) return MLT_ERR_INVALID_ARG;
  if (!(scale == scale) || scale - scale != 0.f) return MLT_ERR_INVALID_ARG;   // NaN or infinite
  if (D != 64 && D != 128) return MLT_ERR_UNSUPPORTED;
  if (B == 0 || H == 0 || Sq == 0) return MLT_OK;
  if (Sk < 1) return MLT_ERR_INVALID_ARG;
  if (!Q || !K || !V || !O) return MLT_ERR_INVALID_ARG;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(Q) || !al16(K) || !al16(V) || !al16(O)) return MLT_ERR_INVALID_ARG;
  if (Sq > INT_MAX || Sk > INT_MAX || B * H > INT_MAX) return MLT_ERR_UNSUPPORTED;
  if (Sk * D * 2 >= ((int64_t)1 << 31)) return MLT_ERR_UNSUPPORTED;   // 32-bit offsets inside one head's K
  return MLT_OK;
}

struct TimedRegion {
  hipStream_t s;
  explicit TimedRegion(hipStream_t st) : s(st) { if (g_ev_start) (void)hipEventRecord(g_ev_start, s); }
  ~TimedRegion() { if (g_ev_stop) (void)hipEventRecord(g_ev_stop, s); }
};

}  // namespace

extern "C" {

int mlt_gemm(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
             int64_t ldb, int transB, void* C, int64_t ldc, int dtype, void* stream) {
  int rc = check_gemm(M, N, K, A, lda, B, ldb, transB, C, ldc, dtype);
  if (rc != MLT_OK) return rc;
  if (M == 0 || N == 0) return MLT_OK;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  GemmArgs g{M, N, K, (const uint16_t*)A, lda, (const uint16_t*)B, ldb, transB ? 1 : 0,
             (uint16_t*)C, ldc, dtype, forced_gemm_variant(), 0};
  g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_gemm(g, p, s);
  }
  if (rc == MLT_OK) note_gemm_kernel(p);
  return rc;
}

int mlt_gemm_noalloc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                     int64_t ldb, int transB, void* C, int64_t ldc, int dtype, void* stream) {
  int rc = check_gemm(M, N, K, A, lda, B, ldb, transB, C, ldc, dtype);
  if (rc != MLT_OK) return rc;
  if (M == 0 || N == 0) return MLT_OK;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  GemmArgs g{M, N, K, (const uint16_t*)A, lda, (const uint16_t*)B, ldb, transB ? 1 : 0,
             (uint16_t*)C, ldc, dtype, forced_gemm_variant(), 0};
  g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
  if (p.parts > 1) {
    if (p.scratch_bytes > kStaticScratchBytes) return MLT_ERR_SCRATCH;
    g.scratch = static_scratch_of_current_device();
    if (!g.scratch) return MLT_ERR_DEVICE;
  }
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_gemm(g, p, s);
  }
  if (rc == MLT_OK) note_gemm_kernel(p);
  return rc;
}

int mlt_gemm_acc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                 int64_t ldb, int transB, float* C, int64_t ldc, int dtype, void* stream) {
  int rc = check_gemm(M, N, K, A, lda, B, ldb, transB, C, ldc, dtype);
  if (rc != MLT_OK) return rc;
  if (M == 0 || N == 0 || K == 0) return MLT_OK;          // C += (empty sum)
  if (reinterpret_cast<uintptr_t>(C) & 3) return MLT_ERR_INVALID_ARG;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  GemmArgs g{M, N, K, (const uint16_t*)A, lda, (const uint16_t*)B, ldb, transB ? 1 : 0,
             (uint16_t*)C, ldc, dtype, forced_gemm_variant(), 1};
  g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_gemm(g, p, s);
  }
  if (rc == MLT_OK) note_gemm_kernel(p);
  return rc;
}

int mlt_gemm_tiled(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                   int64_t ldb, int transB, void* C, int64_t ldc, int dtype, int tiling,
                   void* stream) {
  int rc = check_gemm(M, N, K, A, lda, B, ldb, transB, C, ldc, dtype);
  if (rc != MLT_OK) return rc;
  if (tiling < 0 || tiling > 3) return MLT_ERR_INVALID_ARG;
  if (M == 0 || N == 0) return MLT_OK;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  GemmArgs g{M, N, K, (const uint16_t*)A, lda, (const uint16_t*)B, ldb, transB ? 1 : 0,
             (uint16_t*)C, ldc, dtype, forced_gemm_variant(), 0};
  // horizontal: the wavefronts split the rows of the workgroup tile only; vertical: the columns
  // only; square: 2 x 2 square sub-tiles (the pipelined kernel when the operands allow it)
  if (tiling == 1) g.forced = GEMM_256_W8X1;
  if (tiling == 2) g.forced = GEMM_256_W1X8;
  if (tiling == 3) g.forced = gemm_pp_ok(g) ? GEMM_256_W4 : GEMM_256;
  g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_gemm(g, p, s);
  }
  if (rc == MLT_OK) note_gemm_kernel(p);
  return rc;
}

int mlt_gemm_bias_act(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                      int64_t ldb, int transB, const void* bias, int act, void* C, int64_t ldc,
                      int dtype, void* stream) {
  int rc = check_gemm(M, N, K, A, lda, B, ldb, transB, C, ldc, dtype);
  if (rc != MLT_OK) return rc;
  if (act < 0 || act > 2) return MLT_ERR_INVALID_ARG;
  if (bias && (reinterpret_cast<uintptr_t>(bias) & 1)) return MLT_ERR_INVALID_ARG;
  if (M == 0 || N == 0) return MLT_OK;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  GemmArgs g{M, N, K, (const uint16_t*)A, lda, (const uint16_t*)B, ldb, transB ? 1 : 0,
             (uint16_t*)C, ldc, dtype, forced_gemm_variant(), 0};
  g.bias = (const uint16_t*)bias;
  g.act = act;
  g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_gemm(g, p, s);
  }
  if (rc == MLT_OK) note_gemm_kernel(p);
  return rc;
}

int mlt_mha_fwd(int64_t B, int64_t H, int64_t Sq, int64_t Sk, int64_t D, const void* Q,
                const void* K, const void* V, void* O, float scale, int causal, int dtype,
                void* stream) {
  int rc = check_mha(B, H, Sq, Sk, D, Q, K, V, O, scale, dtype);
  if (rc != MLT_OK) return rc;
  if (B == 0 || H == 0 || Sq == 0) return MLT_OK;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  MhaArgs a{B, H, Sq, Sk, D, (const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V,
            (uint16_t*)O, scale, causal ? 1 : 0, dtype, overrides().mha, overrides().ps_grid};
  MhaPlan p = plan_mha(a);
  if (!p.supported) return MLT_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  {
    TimedRegion t(s);
    rc = run_mha(a, p, s);
  }
  if (rc == MLT_OK) g_last_kernel = p.name;
  return rc;
}

int mlt_paged_attn_decode(int64_t B, int64_t H, int64_t D, int64_t block_size, int64_t max_blocks,
                          int64_t num_blocks, const void* Q, const void* Kc, const void* Vc,
                          const int32_t* block_table, const int32_t* seq_lens, void* O,
                          float scale, int dtype, void* stream) {
  if (dtype != MLT_BF16 && dtype != MLT_FP16) return MLT_ERR_INVALID_ARG;
  if (B < 0 || H < 0 || D <= 0 || block_size <= 0 || max_blocks <= 0 || num_blocks <= 0)
    return MLT_ERR_INVALID_ARG;
  if (!(scale == scale) || scale - scale != 0.f) return MLT_ERR_INVALID_ARG;   // NaN or infinite
  if (D != 64 && D != 128) return MLT_ERR_UNSUPPORTED;
  if (block_size % 16 || block_size > 1024) return MLT_ERR_UNSUPPORTED;
  if (B == 0 || H == 0) return MLT_OK;
  if (!Q || !Kc || !Vc || !block_table || !seq_lens || !O) return MLT_ERR_INVALID_ARG;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(Q) || !al16(Kc) || !al16(Vc)) return MLT_ERR_INVALID_ARG;
  if (B * H > INT_MAX || max_blocks * block_size > INT_MAX || num_blocks > INT_MAX)
    return MLT_ERR_UNSUPPORTED;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  PagedArgs a{B, H, D, block_size, max_blocks, num_blocks, (const uint16_t*)Q, (const uint16_t*)Kc,
              (const uint16_t*)Vc, block_table, seq_lens, (uint16_t*)O, scale, dtype};
  a.forced_split = overrides().key_split;
  hipStream_t s = (hipStream_t)stream;
  int rc, nsplit = 1;
  {
    TimedRegion t(s);
    rc = run_paged_decode(a, s, &nsplit);
  }
  if (rc == MLT_OK) {
    static thread_local char name[48];
    if (nsplit > 1) snprintf(name, sizeof name, "paged_decode_d%d_w4_keysplit%d", (int)D, nsplit);
    else snprintf(name, sizeof name, "paged_decode_d%d_w4", (int)D);
    g_last_kernel = name;
  }
  return rc;
}

static int probe_mfma_impl(int mfma_size, int iters, const void* data, void* sink, double* flop,
                           void* stream) {
  if (iters < 1 || iters > (1 << 20) || !data || !sink || !flop) return MLT_ERR_INVALID_ARG;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  DeviceInfo di;
  if (!device_info(di)) return MLT_ERR_DEVICE;
  const int ncu = di.ncu;
  hipStream_t s = (hipStream_t)stream;
  double f;
  {
    TimedRegion t(s);
    f = run_mfma_probe(iters, ncu, data, (float*)sink, mfma_size, s);
  }
  if (f < 0) return MLT_ERR_LAUNCH;
  *flop = f;
  g_last_kernel = mfma_size == 16 ? "mfma16_rate_probe" : "mfma_rate_probe";
  return MLT_OK;
}

int mlt_probe_mfma(int iters, const void* data, void* sink, double* flop, void* stream) {
  return probe_mfma_impl(32, iters, data, sink, flop, stream);
}

int mlt_probe_mfma16(int iters, const void* data, void* sink, double* flop, void* stream) {
  return probe_mfma_impl(16, iters, data, sink, flop, stream);
}

int mlt_probe_hbm_read(const void* data, int64_t bytes, void* sink, void* stream) {
  if (!data || !sink || bytes < 16 || bytes % 16 != 0 ||
      (reinterpret_cast<uintptr_t>(data) & 15) != 0)
    return MLT_ERR_INVALID_ARG;
  if (!device_is_gfx950()) return MLT_ERR_DEVICE;
  DeviceInfo di;
  if (!device_info(di)) return MLT_ERR_DEVICE;
  const int ncu = di.ncu;
  hipStream_t s = (hipStream_t)stream;
  int rc;
  {
    TimedRegion t(s);
    rc = run_hbm_read_probe(data, bytes, (uint32_t*)sink, ncu, s);
  }
  if (rc == MLT_OK) g_last_kernel = "hbm_read_probe";
  return rc;
}

void mlt_set_timing_events(void* start_event, void* stop_event) {
  g_ev_start = (hipEvent_t)start_event;
  g_ev_stop = (hipEvent_t)stop_event;
}

const char* mlt_last_kernel(void) { return g_last_kernel; }

int mlt_diag_force_variant(const char* gemm_variant, const char* mha_variant) {
  int g = overrides().gemm, m = overrides().mha;
  if (gemm_variant) {
    g = lookup_variant(kGemmVariants, gemm_variant, GEMM_AUTO);
    if (g == -2) return MLT_ERR_INVALID_ARG;
  }
  if (mha_variant) {
    m = lookup_variant(kMhaVariants, mha_variant, MHA_AUTO);
    if (m == -2) return MLT_ERR_INVALID_ARG;
  }
  overrides().gemm = g;
  overrides().mha = m;
  return MLT_OK;
}

int mlt_diag_force_k_parts(int parts) {
  if (parts != 0 && parts != 1 && parts != 2 && parts != 4 && parts != 8) return MLT_ERR_INVALID_ARG;
  overrides().gemm_parts = parts;
  return MLT_OK;
}

int mlt_diag_force_key_split(int ranges) {
  if (ranges < 0 || ranges > 64) return MLT_ERR_INVALID_ARG;
  overrides().key_split = ranges;
  return MLT_OK;
}

int mlt_diag_set_persistent_grid(int workgroups) {
  if (workgroups < 0 || workgroups >= (1 << 20)) return MLT_ERR_INVALID_ARG;
  overrides().ps_grid = workgroups;
  return MLT_OK;
}

int mlt_query_tiling(int op, const int64_t dims[4], int dtype, int32_t out[10]) {
  if (!dims || !out) return MLT_ERR_INVALID_ARG;
  if (dtype != MLT_BF16 && dtype != MLT_FP16) return MLT_ERR_INVALID_ARG;
  if (op == 0) {
    if (dims[0] < 0 || dims[1] < 0 || dims[2] < 0) return MLT_ERR_INVALID_ARG;
    // Alignment is unknown here: assume aligned pointers and tight leading dimensions.
    GemmArgs g{dims[0], dims[1], dims[2], nullptr, dims[2], nullptr, dims[3] ? dims[2] : dims[1],
               dims[3] ? 1 : 0, nullptr, dims[1], dtype, forced_gemm_variant(), 0};
    g.forced_parts = overrides().gemm_parts;
  GemmPlan p = plan_gemm(g);
    if (p.variant == GEMM_ZERO) { for (int i = 0; i < 10; ++i) out[i] = 0; return MLT_OK; }
    out[0] = p.bm; out[1] = p.bn; out[2] = p.wm; out[3] = p.wn;
    out[4] = p.bm / p.wm; out[5] = p.bn / p.wn; out[6] = p.mfma_m; out[7] = p.mfma_n;
    out[8] = p.mfma_k; out[9] = p.bk;
    return MLT_OK;
  }
  if (op == 1) {
    if (dims[0] < 0 || dims[1] < 1) return MLT_ERR_INVALID_ARG;
    if (dims[2] != 64 && dims[2] != 128) return MLT_ERR_UNSUPPORTED;
    MhaArgs a{1, 1, dims[0], dims[1], dims[2], nullptr, nullptr, nullptr, nullptr, 1.f,
              dims[3] ? 1 : 0, dtype, overrides().mha, overrides().ps_grid};
    MhaPlan p = plan_mha(a);
    if (!p.supported) return MLT_ERR_UNSUPPORTED;
    out[0] = p.bm; out[1] = (int32_t)dims[2]; out[2] = p.waves; out[3] = 1;
    out[4] = p.bm / p.waves; out[5] = (int32_t)dims[2];
    out[6] = p.mfma_size; out[7] = p.mfma_size; out[8] = p.mfma_size == 16 ? 32 : 16;
    out[9] = p.bn;
    return MLT_OK;
  }
  return MLT_ERR_INVALID_ARG;
}

const char* mlt_status_string(int status) {
  switch (status) {
    case MLT_OK: return "ok";
    case MLT_ERR_INVALID_ARG: return "invalid argument";
    case MLT_ERR_UNSUPPORTED: return "unsupported configuration";
    case MLT_ERR_LAUNCH: return "kernel launch failed";
    case MLT_ERR_DEVICE: return "no usable gfx950 device";
    case MLT_ERR_SCRATCH: return "the call needs more scratch memory than the no-allocation entry point has";
  }
  return "unknown status";
}

const char* mlt_version(void) { return "0.1.0"; }

}  // extern "C"
