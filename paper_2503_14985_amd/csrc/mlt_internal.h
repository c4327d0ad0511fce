// Host-side plumbing shared by the entry points and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mlt {

enum GemmVariant {
  GEMM_AUTO = -1, GEMM_ZERO = 0, GEMM_GENERAL = 1,
  GEMM_256 = 2,       // 256x256x64, 4 wavefronts (2x2) of 128x128 (tiling hint "square" with a ragged K)
  GEMM_256_W8 = 4,    // 256x256x64, 8 wavefronts (2x4) of 128x64 (big tiles when the direct loads do not apply)
  GEMM_SKINNY = 7,    // M <= 64, B stored N x K: 16 columns per workgroup, K split over 8 wavefronts
  GEMM_SKINNY_DMA = 8,  // same shapes, B streamed through an LDS ring: 16 columns x 512 k per stage
  GEMM_256_W4 = 10,   // 256x256x64, 4 wavefronts (2x2) of 128x128, software-pipelined, direct-to-LDS loads
  GEMM_256_PP16 = 11, // 256x256x64, 8 wavefronts (2x4), two-group schedule, direct-to-LDS loads, 16x16x32 MFMAs
  GEMM_256_W8X1 = 12, // 256x256x64, 8 wavefronts as 8x1: row strips of 32 x 256 ("horizontal")
  GEMM_256_W1X8 = 13, // 256x256x64, 8 wavefronts as 1x8: column strips of 256 x 32 ("vertical")
  GEMM_128_W8 = 14,   // 128x128x64, 8 wavefronts (2x4) of 64x32
  GEMM_64X128_W8 = 15, // 64x128x64, 8 wavefronts (2x4) of 32x32
  GEMM_64_W4 = 16,    // 64x64x64, 4 wavefronts (2x2) of 32x32
  GEMM_128_K2 = 17,   // 128x128x64, 2 groups of 8 wavefronts, each group half of the K steps
  GEMM_64X128_K2 = 18, // 64x128x64, 2 groups of 8 wavefronts
  GEMM_64_K4 = 19,    // 64x64x64, 4 groups of 4 wavefronts (3 when B is K x N), each group its share of the K steps
  GEMM_128_PP16 = 20, // 128x128x64, 8 wavefronts (2x4) of 64x32, two-group schedule, direct-to-LDS loads, two workgroups per CU
  GEMM_128_PP16_K128 = 21, // the same tile with K steps of 128 (one workgroup per CU, phases of twice the length)
  GEMM_NUM_VARIANTS
};

struct GemmArgs {
  int64_t M, N, K;
  const uint16_t* A; int64_t lda;
  const uint16_t* B; int64_t ldb; int transB;
  uint16_t* C; int64_t ldc;
  int dtype;
  int forced;  // GemmVariant or GEMM_AUTO
  int acc32;   // 0: C is 16-bit and overwritten; 1: C is fp32 and accumulated into (C += A*B)
  const uint16_t* bias = nullptr;  // N elements of the input type added to every row (16-bit C only), or null
  int act = 0;                     // 0 none, 1 relu, 2 gelu: applied after the bias (16-bit C only)
  // K split across workgroups: the fp32 scratch the partial products go to (parts * M * N floats)
  // and the number of parts the plan asks for; run_gemm fills both in.
  float* scratch = nullptr;
  int parts = 1;
  int64_t scratch_limit = -1;      // plan_gemm: largest scratch (bytes) a split may use; -1 = no limit
  int forced_parts = 0;            // plan_gemm: 0 = the cost model's choice, 1 / 2 / 4 / 8 = forced
  int epi() const { return acc32 ? 1 : (act << 1); }   // the kernels' epilogue word
  bool fused() const { return bias != nullptr || act != 0; }
};

struct GemmPlan {
  int variant = GEMM_GENERAL;
  int parts = 1;                   // > 1: K split across workgroups, partial products through a scratch
  int64_t scratch_bytes = 0;       // parts * M * N * 4 when parts > 1
  const char* name = "";
  int bm = 0, bn = 0, bk = 0, wm = 0, wn = 0;
  int mfma_m = 32, mfma_n = 32, mfma_k = 16;
};

// mlt_gemm_noalloc: bytes of the fixed device array that takes the partial products of a K split
// across workgroups (no plan the library makes by itself needs more than half of it), and that
// array's address on the current device (nullptr if it cannot be had)
constexpr int64_t kStaticScratchBytes = (int64_t)32 << 20;
float* static_scratch_of_current_device();

GemmPlan plan_gemm(const GemmArgs& g);
int run_gemm(const GemmArgs& g, GemmPlan& p, hipStream_t s);
bool gemm_pp_ok(const GemmArgs& g);            // gemm_pp.hip: can the two-group kernel take this problem?
int run_gemm_pp(const GemmArgs& g, int tile, int kstep, hipStream_t s);   // tile: 256 or 128; K step 64 or (tile 128 only) 128
int run_gemm_w4(const GemmArgs& g, hipStream_t s);   // gemm_w4.hip; same operand requirements (gemm_pp_ok)
bool gemm_skinny_ok(const GemmArgs& g);        // gemm_skinny.hip
int run_gemm_skinny(const GemmArgs& g, hipStream_t s);
bool gemm_skinny_dma_ok(const GemmArgs& g);
int run_gemm_skinny_dma(const GemmArgs& g, hipStream_t s);

enum MhaVariant {
  MHA_AUTO = -1,
  MHA_PP32 = 0,   // two-group kernel, 32x32x16 MFMAs, one workgroup per (batch*head, query tile)
  MHA_PP16 = 1,   // the same on 16x16x32 MFMAs
  MHA_PS = 2,     // persistent form of the two-group kernel (unmasked, D = 128, at least two key tiles)
  MHA_NUM_VARIANTS
};

struct MhaArgs {
  int64_t B, H, Sq, Sk, D;
  const uint16_t *Q, *K, *V;
  uint16_t* O;
  float scale;
  int causal, dtype;
  int forced = MHA_AUTO;   // MhaVariant or MHA_AUTO
  int ps_grid = 0;         // persistent kernel: number of workgroups (0: one per CU)
};

struct MhaPlan {
  const char* name = "";
  int bm = 0, bn = 0, waves = 0;
  bool supported = false;
  int mfma_size = 32;       // 32 = 32x32x16 MFMAs, 16 = 16x16x32
  bool persistent = false;  // one workgroup per CU walking through the items
};
bool mha_pp_ok(const MhaArgs& a);
int run_mha_pp(const MhaArgs& a, int mfma_size, hipStream_t s);
bool mha_ps_ok(const MhaArgs& a);              // mha_pp.hip: can the persistent kernel take this problem?
int run_mha_ps(const MhaArgs& a, hipStream_t s);

// Process-wide overrides of the automatic kernel choice, for tuning and for the tests that must
// reach every kernel (mlt_diag_force_variant; initial values from MLT_GEMM_VARIANT /
// MLT_MHA_VARIANT / MLT_MHA_PS_GRID, read once).
struct Overrides { int gemm = GEMM_AUTO; int gemm_parts = 0; int mha = MHA_AUTO; int ps_grid = 0; int key_split = 0; };
Overrides& overrides();
// Device facts the launchers need, cached per thread for the current device.
struct DeviceInfo { int ncu = 0; int nxcd = 0; bool gfx950 = false; };
bool device_info(DeviceInfo& out);
// XCDs of the current device (hipDeviceAttributeNumberOfXccs; 8, the MI355X's, if it cannot be
// read). Only the workgroup -> tile maps use it: a wrong value costs L2 hits, never correctness.
int device_xcds();

// probe.hip: launches the register-only MFMA loop, returns the flop it will execute (< 0: launch failed)
double run_mfma_probe(int iters, int nblocks, const void* data, float* sink, int mfma_size, hipStream_t s);
int run_hbm_read_probe(const void* data, int64_t bytes, uint32_t* sink, int ncu, hipStream_t s);

MhaPlan plan_mha(const MhaArgs& a);
int run_mha(const MhaArgs& a, const MhaPlan& p, hipStream_t s);

struct PagedArgs {
  int64_t B, H, D, block_size, max_blocks, num_blocks;
  const uint16_t *Q, *Kc, *Vc;
  const int32_t *block_table, *seq_lens;
  uint16_t* O;
  float scale;
  int dtype;
  int forced_split = 0;      // > 0: ranges of keys per (sequence, head), from mlt_diag_force_key_split
};
// paged.hip; *nsplit_out: the number of key ranges per (sequence, head) that ran
int run_paged_decode(const PagedArgs& a, hipStream_t s, int* nsplit_out);

// The library's own scratch memory for a stream of the current device: at least `bytes`, kept
// (and grown by doubling) from call to call, never freed; nullptr if it cannot be had. Work of
// one stream that uses it is ordered by the stream.
float* cached_scratch(int64_t bytes, hipStream_t s);

}  // namespace mlt
