// GEMM C = A*B for gfx950: 16-bit inputs, fp32 accumulation on MFMA, 16-bit output.
//
// The paper (arXiv 2503.14985, Section 2) splits the GEMM in three levels: a workgroup tile of C
// (Listing 1), a square partition of that tile over the warps (Section 2.1: warpsPerCTA and
// sizePerWarp), and the split of each warp's dot into hardware-sized dots (Section 2.3). The
// kernels here have the same three levels, fixed by template parameters and re-derived for CDNA4:
//   workgroup tile BM x BN, K step BK            (paper: 256 x 256, K step 32)
//   WM x WN wavefronts, each owning (BM/WM) x (BN/WN)   (paper: 8 x 4 warps of 32 x 64)
//   MFMA 32x32x16 tiles inside the wavefront tile       (paper: 8x16x16 DPAS)
// Unlike the paper's target there is no 2-D block load from memory into registers, so operand
// tiles are staged through LDS: each byte is fetched from global memory once per workgroup and
// read by the wavefronts that share it (the rows/columns of the warp grid that Section 2.2 notes
// work on the same sub-block of A or B).
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

// ------------------------------------------------------------------------------------------
// Workgroup id -> C tile. Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each
// with its own L2. First undo that so every XCD owns one contiguous range of logical ids, then
// walk logical ids in column-major order inside bands of GROUP_M tile rows, so that the
// workgroups resident on one XCD at a time share A row panels and B column panels.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void tile_of_block(int bid, int nbm, int nbn, int& tm, int& tn) {
  constexpr int NXCD = 8, GROUP_M = 8;
  const int total = nbm * nbn;
  const int q = total / NXCD, rem = total % NXCD;
  const int xcd = bid % NXCD, idx = bid / NXCD;
  const int logical = xcd * q + (xcd < rem ? xcd : rem) + idx;
  const int per_group = GROUP_M * nbn;
  const int g = logical / per_group;
  const int first_m = g * GROUP_M;
  const int rows = (nbm - first_m) < GROUP_M ? (nbm - first_m) : GROUP_M;
  const int in_g = logical % per_group;
  tm = first_m + in_g % rows;
  tn = in_g / rows;
}

// ------------------------------------------------------------------------------------------
// Main kernel. Requirements checked by the host: K % 8 == 0, lda % 8 == 0, ldb % 8 == 0,
// N % 8 == 0 when B is K x N row-major, A and B 16-byte aligned. M, N and K need not be
// multiples of the tile: out-of-range rows are clamped on load (their products land in
// accumulator rows/columns that are never stored) and the K tail is zero-filled.
//
// LDS layout per stage (elements are 16-bit):
//   A tile   [BM][BK + 8]          k contiguous; the 16-byte pad makes the row stride 36 dwords,
//                                  so 16 consecutive rows at one k offset fall in 16 distinct
//                                  4-bank groups of the 64 banks
//   B tile   TRANSB:  [BN][BK + 8] same as A (global B is N x K, k contiguous)
//            !TRANSB: [BK][BN + 32] n contiguous, as in global memory; fragments are fetched with
//                                  the transposing LDS read; the 64-byte pad puts the 4 k-rows of
//                                  a 16-lane read group into disjoint bank ranges
// Two stages; global loads for step k+1 are issued before the MFMAs of step k, parked in
// registers and written to the other stage afterwards, one barrier per step.
// ------------------------------------------------------------------------------------------
template <typename Tag, int BM, int BN, int BK, int WM, int WN, bool TRANSB>
struct GemmTile {
  static constexpr int NT = WM * WN * 64;
  static constexpr int KC = BK / 8;                     // 16-byte chunks along k
  static constexpr int LDA_S = BK + 8;
  static constexpr int A_BYTES = BM * LDA_S * 2;
  static constexpr int LDB_S = TRANSB ? BK + 8 : BN + 32;
  static constexpr int B_BYTES = (TRANSB ? BN : BK) * LDB_S * 2;
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int SMEM = 2 * STAGE;
  static constexpr int NA = BM * KC / NT;               // chunks per thread per stage
  static constexpr int NB = BN * KC / NT;
  static constexpr int TM = BM / WM / 32;               // MFMA tiles per wavefront
  static constexpr int TN = BN / WN / 32;
  static_assert(BM * KC % NT == 0 && BN * KC % NT == 0, "tile must split evenly over threads");
  static_assert(BK % 16 == 0 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "MFMA tiling");
};

template <typename Tag, int BM, int BN, int BK, int WM, int WN, bool TRANSB>
__global__ __launch_bounds__(WM* WN * 64, 1) void gemm_tile_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc, int nbm,
    int nbn) {
  typedef GemmTile<Tag, BM, BN, BK, WM, WN, TRANSB> Cfg;
  typedef typename Elem<Tag>::vec8 V8;
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, nbm, nbn, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- per-thread staging assignments (fixed for the whole K loop)
  const uint16_t* a_src[Cfg::NA];
  int a_dst[Cfg::NA], a_k[Cfg::NA];
#pragma unroll
  for (int i = 0; i < Cfg::NA; ++i) {
    const int c = tid + i * Cfg::NT;
    const int row = c / Cfg::KC, kc = c % Cfg::KC;
    int grow = m0 + row;
    grow = grow < M ? grow : M - 1;
    a_src[i] = A + (int64_t)grow * lda + kc * 8;
    a_dst[i] = (row * Cfg::LDA_S + kc * 8) * 2;
    a_k[i] = kc * 8;
  }
  const uint16_t* b_src[Cfg::NB];
  int b_dst[Cfg::NB], b_k[Cfg::NB];
#pragma unroll
  for (int i = 0; i < Cfg::NB; ++i) {
    const int c = tid + i * Cfg::NT;
    if (TRANSB) {
      const int row = c / Cfg::KC, kc = c % Cfg::KC;
      int grow = n0 + row;
      grow = grow < N ? grow : N - 1;
      b_src[i] = B + (int64_t)grow * ldb + kc * 8;
      b_dst[i] = Cfg::A_BYTES + (row * Cfg::LDB_S + kc * 8) * 2;
      b_k[i] = kc * 8;
    } else {
      constexpr int NC = BN / 8;                        // chunks along n
      const int krow = c / NC, nc = c % NC;
      const int gcol = n0 + nc * 8;
      // N % 8 == 0: a chunk is all in or all out; an outside chunk reads column 0 instead
      b_src[i] = B + (int64_t)krow * ldb + (gcol < N ? gcol : 0);
      b_dst[i] = Cfg::A_BYTES + (krow * Cfg::LDB_S + nc * 8) * 2;
      b_k[i] = krow;
    }
  }

  u32x4 ga[Cfg::NA], gb[Cfg::NB];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  // Loads never branch: a chunk outside the matrix re-reads a valid address (row clamp above,
  // column 0 / k 0 here); only chunks past K, which would pollute real outputs, are zeroed.
  auto load_global = [&](int k0, bool tail) {
#pragma unroll
    for (int i = 0; i < Cfg::NA; ++i) {
      const bool ok = !tail || (k0 + a_k[i] < K);
      const u32x4 v = *reinterpret_cast<const u32x4*>(a_src[i] + (ok ? k0 : -a_k[i]));
      ga[i] = ok ? v : zero4;
    }
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) {
      const bool ok = !tail || (k0 + b_k[i] < K);
      u32x4 v;
      if (TRANSB) {
        v = *reinterpret_cast<const u32x4*>(b_src[i] + (ok ? k0 : -b_k[i]));
      } else {
        v = *reinterpret_cast<const u32x4*>(b_src[i] + (ok ? (int64_t)k0 * ldb : -(int64_t)b_k[i] * ldb));
      }
      gb[i] = ok ? v : zero4;
    }
  };
  auto store_lds = [&](int stage) {
    char* base = smem + stage * Cfg::STAGE;
#pragma unroll
    for (int i = 0; i < Cfg::NA; ++i) *reinterpret_cast<u32x4*>(base + a_dst[i]) = ga[i];
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) *reinterpret_cast<u32x4*>(base + b_dst[i]) = gb[i];
  };

  // ---- fragment addresses inside a stage
  // A fragment: row = wavefront row offset + 32*tm + lane%32, 8 consecutive k starting at
  // 8*(lane/32) inside each 16-wide k slice.
  const int a_frag = ((wm * (BM / WM) + (lane & 31)) * Cfg::LDA_S + 8 * (lane >> 5)) * 2;
  int b_frag;
  if (TRANSB) {
    b_frag = Cfg::A_BYTES + ((wn * (BN / WN) + (lane & 31)) * Cfg::LDB_S + 8 * (lane >> 5)) * 2;
  } else {
    // Transposing read: 16-lane group g = lane/16 serves columns 16*(g%2).. of the 32-wide tile
    // and k slots 8*(g/2)..; inside the group, lane s addresses k row s/4, columns 4*(s%4)..
    const int g = lane >> 4, s = lane & 15;
    const int krow = 8 * (g >> 1) + (s >> 2);
    const int col = wn * (BN / WN) + 16 * (g & 1) + 4 * (s & 3);
    b_frag = Cfg::A_BYTES + (krow * Cfg::LDB_S + col) * 2;
  }

  f32x16 acc[Cfg::TM][Cfg::TN];
#pragma unroll
  for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = (K + BK - 1) / BK;
  const bool ragged_k = (K % BK) != 0;                  // only the last step can be partial
  load_global(0, ragged_k && KT == 1);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) load_global((kt + 1) * BK, ragged_k && kt + 2 == KT);
    const char* st = smem + cur * Cfg::STAGE;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      V8 af[Cfg::TM], bf[Cfg::TN];
#pragma unroll
      for (int i = 0; i < Cfg::TM; ++i)
        af[i] = lds_read8<V8>(st, a_frag + (i * 32 * Cfg::LDA_S + kk * 16) * 2);
#pragma unroll
      for (int j = 0; j < Cfg::TN; ++j) {
        if (TRANSB) {
          bf[j] = lds_read8<V8>(st, b_frag + (j * 32 * Cfg::LDB_S + kk * 16) * 2);
        } else {
          const int off = b_frag + (kk * 16 * Cfg::LDB_S + j * 32) * 2;
          s16x4 lo = lds_read_tr4(st, off);
          s16x4 hi = lds_read_tr4(st, off + 4 * Cfg::LDB_S * 2);
          bf[j] = join_tr<V8>(lo, hi);
        }
      }
#pragma unroll
      for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) acc[i][j] = mfma32(af[i], bf[j], acc[i][j]);
    }
    if (more) store_lds(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: fp32 -> 16-bit (RNE), guarded element stores
  const int row_base = m0 + wm * (BM / WM) + 4 * (lane >> 5);
  const int col_base = n0 + wn * (BN / WN) + (lane & 31);
#pragma unroll
  for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
    for (int j = 0; j < Cfg::TN; ++j) {
      const int col = col_base + j * 32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
        if (row < M && col < N) C[(int64_t)row * ldc + col] = Elem<Tag>::from_f32(acc[i][j][r]);
      }
    }
}

// ------------------------------------------------------------------------------------------
// General kernel: any M, N, K, leading dimensions and alignment. 64 x 64 x 32 tile, 4 wavefronts
// of 32 x 32, element-wise guarded loads with zero fill, B always staged as [n][k].
// ------------------------------------------------------------------------------------------
template <typename Tag>
__global__ __launch_bounds__(256) void gemm_general_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, int transB, uint16_t* __restrict__ C,
    int64_t ldc) {
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int BM = 64, BN = 64, BK = 32, LDS_S = BK + 8;
  __shared__ __align__(16) uint16_t As[BM * LDS_S];
  __shared__ __align__(16) uint16_t Bs[BN * LDS_S];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;

  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < BM * BK / 256; ++i) {
      const int e = tid + i * 256;
      const int row = e / BK, k = e % BK;               // consecutive lanes: consecutive k
      const bool ok = (m0 + row < M) && (k0 + k < K);
      As[row * LDS_S + k] = ok ? A[(int64_t)(m0 + row) * lda + k0 + k] : (uint16_t)0;
    }
#pragma unroll
    for (int i = 0; i < BN * BK / 256; ++i) {
      const int e = tid + i * 256;
      int n, k;
      if (transB) { n = e / BK; k = e % BK; } else { k = e / BN; n = e % BN; }
      const bool ok = (n0 + n < N) && (k0 + k < K);
      uint16_t v = 0;
      if (ok) v = transB ? B[(int64_t)(n0 + n) * ldb + k0 + k] : B[(int64_t)(k0 + k) * ldb + n0 + n];
      Bs[n * LDS_S + k] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int off = kk * 16 + 8 * (lane >> 5);
      V8 a = *reinterpret_cast<const V8*>(&As[(wm * 32 + (lane & 31)) * LDS_S + off]);
      V8 b = *reinterpret_cast<const V8*>(&Bs[(wn * 32 + (lane & 31)) * LDS_S + off]);
      acc = mfma32(a, b, acc);
    }
    __syncthreads();
  }
  const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (row < M && col < N) C[(int64_t)row * ldc + col] = Elem<Tag>::from_f32(acc[r]);
  }
}

// K == 0: the empty sum.
__global__ void gemm_zero_kernel(int M, int N, uint16_t* __restrict__ C, int64_t ldc) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < (int64_t)M * N) C[(e / N) * ldc + (e % N)] = 0;
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
template <typename Tag, int BM, int BN, int BK, int WM, int WN, bool TRANSB>
static int launch_tile(const GemmArgs& g, hipStream_t s) {
  typedef GemmTile<Tag, BM, BN, BK, WM, WN, TRANSB> Cfg;
  auto kern = gemm_tile_kernel<Tag, BM, BN, BK, WM, WN, TRANSB>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            Cfg::SMEM) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nbm = (int)((g.M + BM - 1) / BM), nbn = (int)((g.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(nbm * nbn), dim3(Cfg::NT), Cfg::SMEM, s, (int)g.M, (int)g.N,
                     (int)g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc, nbm, nbn);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

template <typename Tag>
static int launch_general(const GemmArgs& g, hipStream_t s) {
  dim3 grid((unsigned)((g.N + 63) / 64), (unsigned)((g.M + 63) / 64));
  hipLaunchKernelGGL(gemm_general_kernel<Tag>, grid, dim3(256), 0, s, (int)g.M, (int)g.N, (int)g.K,
                     g.A, g.lda, g.B, g.ldb, g.transB, g.C, g.ldc);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

static bool fast_path_ok(const GemmArgs& g) {
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(g.A) || !al16(g.B)) return false;
  if (g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
  if (!g.transB && g.N % 8) return false;
  return true;
}

GemmPlan plan_gemm(const GemmArgs& g) {
  GemmPlan p;
  if (g.K == 0) { p.variant = GEMM_ZERO; p.name = "gemm_zero"; return p; }
  if (!fast_path_ok(g) || g.forced == GEMM_GENERAL) {
    p.variant = GEMM_GENERAL; p.name = "gemm_general_64x64x32";
    p.bm = 64; p.bn = 64; p.bk = 32; p.wm = 2; p.wn = 2;
    return p;
  }
  // Big tile when it still fills the chip, otherwise the small one.
  const int64_t tiles256 = ((g.M + 255) / 256) * ((g.N + 255) / 256);
  int v = tiles256 >= 192 ? GEMM_256 : GEMM_128;
  if (g.forced == GEMM_256 || g.forced == GEMM_128) v = g.forced;
  p.variant = v;
  if (v == GEMM_256) { p.bm = 256; p.bn = 256; p.bk = 64; p.wm = 2; p.wn = 2; p.name = g.transB ? "gemm_nt_256x256x64" : "gemm_nn_256x256x64"; }
  else { p.bm = 128; p.bn = 128; p.bk = 64; p.wm = 2; p.wn = 2; p.name = g.transB ? "gemm_nt_128x128x64" : "gemm_nn_128x128x64"; }
  return p;
}

template <typename Tag>
static int run_gemm_t(const GemmArgs& g, const GemmPlan& p, hipStream_t s) {
  switch (p.variant) {
    case GEMM_ZERO: {
      const int64_t n = g.M * g.N;
      hipLaunchKernelGGL(gemm_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                         (int)g.M, (int)g.N, g.C, g.ldc);
      return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
    }
    case GEMM_GENERAL: return launch_general<Tag>(g, s);
    case GEMM_256:
      return g.transB ? launch_tile<Tag, 256, 256, 64, 2, 2, true>(g, s)
                      : launch_tile<Tag, 256, 256, 64, 2, 2, false>(g, s);
    case GEMM_128:
      return g.transB ? launch_tile<Tag, 128, 128, 64, 2, 2, true>(g, s)
                      : launch_tile<Tag, 128, 128, 64, 2, 2, false>(g, s);
  }
  return MLT_ERR_UNSUPPORTED;
}

int run_gemm(const GemmArgs& g, const GemmPlan& p, hipStream_t s) {
  return g.dtype == MLT_BF16 ? run_gemm_t<bf16_tag>(g, p, s) : run_gemm_t<f16_tag>(g, p, s);
}

}  // namespace mlt
