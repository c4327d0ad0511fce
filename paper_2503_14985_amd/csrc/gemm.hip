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
#include <mutex>

#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

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
  static_assert(NT % KC == 0 && NT % (BN / 8) == 0, "a thread's chunks must share their column");
  static_assert(BK % 16 == 0 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "MFMA tiling");
};

// K split across workgroups (part_steps > 0): the grid's y index is the part; part p takes the K
// steps p * part_steps .. of the problem and stores its fp32 partial tile (epi = EPI_PART32) into
// slice p of the scratch that C_ then points at (slices part_stride floats apart, row stride ldc);
// gemm_splitk_reduce_kernel adds the slices in a fixed order and applies the real epilogue.
template <typename Tag, int BM, int BN, int BK, int WM, int WN, bool TRANSB, int KS>
__global__ __launch_bounds__(WM* WN * 64 * KS) void gemm_tile_kernel(
    int M, int N, int K_, const uint16_t* __restrict__ A_, int64_t lda,
    const uint16_t* __restrict__ B_, int64_t ldb, uint16_t* __restrict__ C_, int64_t ldc, int nbm,
    int nbn, int nxcd, int epi, const uint16_t* __restrict__ bias, int part_steps, int64_t part_stride) {
  typedef GemmTile<Tag, BM, BN, BK, WM, WN, TRANSB> Cfg;
  typedef typename Elem<Tag>::vec8 V8;
  extern __shared__ __align__(16) char smem_all[];
  const uint16_t* A = A_;
  const uint16_t* B = B_;
  uint16_t* C = C_;
  int K = K_;
  if (part_steps > 0) {
    const int part = blockIdx.y;
    const int k_begin = part * part_steps * BK;            // < K_: the host launches no empty part
    A += k_begin;
    B += TRANSB ? (int64_t)k_begin : (int64_t)k_begin * ldb;
    K = K_ - k_begin < part_steps * BK ? K_ - k_begin : part_steps * BK;
    C = reinterpret_cast<uint16_t*>(reinterpret_cast<float*>(C_) + (int64_t)part * part_stride);
  }

  // KS > 1: the workgroup holds KS groups of WM x WN wavefronts; group kg runs the whole pipeline
  // below on its own LDS stages over its own share of the K steps, and the groups' accumulators
  // are added through LDS at the end (see there). tid, wave: inside the group.
  const int kg = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / Cfg::NT);
  const int tid = KS == 1 ? (int)threadIdx.x : (int)threadIdx.x % Cfg::NT;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  char* const smem = smem_all + kg * Cfg::SMEM;
  int tile_m, tile_n;
  tile_of_block<8>(blockIdx.x, nbm, nbn, nxcd, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- per-thread staging assignments (fixed for the whole K loop)
  // Chunk c = tid + i*NT of a [rows][KC] tile is (row c / KC, k chunk c % KC). NT is a multiple of
  // KC, so the k chunk is the same for every i and row_i = row_0 + i * (NT / KC): LDS offsets
  // differ by compile-time constants and only the clamped global row pointers are per-i values.
  constexpr int RSTEP = Cfg::NT / Cfg::KC;              // tile rows between a thread's chunks
  const int st_row = tid / Cfg::KC, st_k = (tid % Cfg::KC) * 8;
  const uint16_t* a_src[Cfg::NA];
#pragma unroll
  for (int i = 0; i < Cfg::NA; ++i) {
    int grow = m0 + st_row + i * RSTEP;
    grow = grow < M ? grow : M - 1;
    a_src[i] = A + (int64_t)grow * lda + st_k;
  }
  const int a_dst = (st_row * Cfg::LDA_S + st_k) * 2;
  constexpr int A_DST_STEP = RSTEP * Cfg::LDA_S * 2;

  const uint16_t* b_src[TRANSB ? Cfg::NB : 1];
  int b_dst, b_k;
  constexpr int NC = BN / 8;                            // 16-byte chunks along n (row-major B)
  constexpr int KSTEP = Cfg::NT / NC;                   // k rows between a thread's chunks
  constexpr int B_DST_STEP = (TRANSB ? RSTEP : KSTEP) * Cfg::LDB_S * 2;
  if (TRANSB) {
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) {
      int grow = n0 + st_row + i * RSTEP;
      grow = grow < N ? grow : N - 1;
      b_src[i] = B + (int64_t)grow * ldb + st_k;
    }
    b_dst = Cfg::A_BYTES + (st_row * Cfg::LDB_S + st_k) * 2;
    b_k = st_k;
  } else {
    const int krow = tid / NC, nc = tid % NC;
    const int gcol = n0 + nc * 8;
    // N % 8 == 0: a chunk is all in or all out; an outside chunk reads column 0 instead
    b_src[0] = B + (int64_t)krow * ldb + (gcol < N ? gcol : 0);
    b_dst = Cfg::A_BYTES + (krow * Cfg::LDB_S + nc * 8) * 2;
    b_k = krow;
  }

  u32x4 ga[Cfg::NA], gb[Cfg::NB];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  // Loads never branch per element: a chunk outside the matrix re-reads a valid address (row
  // clamp above, column 0 here). Only the last K step can run past K; it takes the second form,
  // which re-reads k = 0 for chunks past K and zeroes them (they would pollute real outputs).
  auto load_global_full = [&](int k0) {
#pragma unroll
    for (int i = 0; i < Cfg::NA; ++i) ga[i] = *reinterpret_cast<const u32x4_mem*>(a_src[i] + k0);
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) {
      if (TRANSB) gb[i] = *reinterpret_cast<const u32x4_mem*>(b_src[i] + k0);
      else gb[i] = *reinterpret_cast<const u32x4_mem*>(b_src[0] + (int64_t)(k0 + i * KSTEP) * ldb);
    }
  };
  auto load_global_tail = [&](int k0) {
#pragma unroll
    for (int i = 0; i < Cfg::NA; ++i) {
      const bool ok = k0 + st_k < K;
      const u32x4 v = *reinterpret_cast<const u32x4_mem*>(a_src[i] + (ok ? k0 : -st_k));
      ga[i] = ok ? v : zero4;
    }
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) {
      if (TRANSB) {
        const bool ok = k0 + b_k < K;
        const u32x4 v = *reinterpret_cast<const u32x4_mem*>(b_src[i] + (ok ? k0 : -b_k));
        gb[i] = ok ? v : zero4;
      } else {
        const int kr = k0 + i * KSTEP;                  // + b_k = the k row of this chunk
        const bool ok = kr + b_k < K;
        const u32x4 v = *reinterpret_cast<const u32x4_mem*>(b_src[0] + (int64_t)(ok ? kr : -b_k) * ldb);
        gb[i] = ok ? v : zero4;
      }
    }
  };
  auto load_global = [&](int k0, bool tail) {
    if (tail) load_global_tail(k0); else load_global_full(k0);
  };
  auto store_lds = [&](int stage) {
    char* base = smem + stage * Cfg::STAGE;
#pragma unroll
    for (int i = 0; i < Cfg::NA; ++i) *reinterpret_cast<u32x4_mem*>(base + a_dst + i * A_DST_STEP) = ga[i];
#pragma unroll
    for (int i = 0; i < Cfg::NB; ++i) *reinterpret_cast<u32x4_mem*>(base + b_dst + i * B_DST_STEP) = gb[i];
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

  // Fragments of k slice kk of a stage: TM A operands and TN B operands.
  auto load_frags = [&](const char* st, int kk, V8 (&af)[Cfg::TM], V8 (&bf)[Cfg::TN]) {
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
  };

  const int KT = (K + BK - 1) / BK;
  const bool ragged_k = (K % BK) != 0;                  // only the last step can be partial
  constexpr int NKK = BK / 16;
  static_assert(NKK == 4, "the schedule below is written for four k slices per stage");
  // This group's K steps: kg, kg + KS, kg + 2 KS, ... (all of them when KS == 1), so that at any
  // time the groups of a workgroup read neighbouring pieces of the same operand rows (with the
  // operands stored k-contiguous: KS x 128 contiguous bytes of every row instead of KS pieces far
  // apart); every group runs the loop KTG times so that all wavefronts meet at the same barriers,
  // idle once its steps are done.
  const int KTG = (KT + KS - 1) / KS;
  const int kt_begin = kg;
  const int kt_end = KT;
  auto load_tile = [&](int t) { load_global(t * BK, ragged_k && t == KT - 1); };

  // Software pipeline. Stage s holds the group's i-th tile (s = i & 1). During step kt:
  //   slice 0: read fragments of slice 1 | MFMAs of slice 0
  //   slice 1: read fragments of slice 2 | MFMAs of slice 1 | write tile kt+1 (already in
  //            registers since the previous step) to the other stage | issue the global loads
  //            of tile kt+2 into the registers just freed
  //   slice 2: read fragments of slice 3 | MFMAs of slice 2 | barrier
  //   slice 3: read fragments of slice 0 of tile kt+1 | MFMAs of slice 3
  // The barrier sits where every wavefront has issued its last read of stage s and its writes
  // of tile kt+1, so after it stage s may be overwritten (in step kt+1) and tile kt+1 may be
  // read; its latency and that of the first fragment reads hide behind the MFMAs of slice 3.
  const bool any = kt_begin < kt_end;
  if (any) {
    load_tile(kt_begin);
    store_lds(0);
    if (kt_begin + KS < kt_end) load_tile(kt_begin + KS);
  }
  __syncthreads();

  V8 af[2][Cfg::TM], bf[2][Cfg::TN];
  if (any) load_frags(smem, 0, af[0], bf[0]);

  auto mfma_slice = [&](int which) {
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
      for (int j = 0; j < Cfg::TN; ++j)
        acc[i][j] = mfma32(af[which][i], bf[which][j], acc[i][j]);
  };

  for (int it = 0; it < KTG; ++it) {
    const int kt = kt_begin + it * KS;
    const bool active = KS == 1 || kt < kt_end;
    const int cur = it & 1;
    const char* st = smem + cur * Cfg::STAGE;
    const char* nx = smem + (cur ^ 1) * Cfg::STAGE;
    const bool have_next = kt + KS < kt_end;

    if (active) {
      load_frags(st, 1, af[1], bf[1]);
      __builtin_amdgcn_sched_barrier(0);
      mfma_slice(0);
      __builtin_amdgcn_sched_barrier(0);

      load_frags(st, 2, af[0], bf[0]);
      __builtin_amdgcn_sched_barrier(0);
      mfma_slice(1);
      __builtin_amdgcn_sched_barrier(0);
      if (have_next) {
        store_lds(cur ^ 1);
        if (kt + 2 * KS < kt_end) load_tile(kt + 2 * KS);
      }
      __builtin_amdgcn_sched_barrier(0);

      load_frags(st, 3, af[1], bf[1]);
      __builtin_amdgcn_sched_barrier(0);
      mfma_slice(0);                                    // slice 2 lives in fragment set 0
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();

    if (active) {
      if (have_next) load_frags(nx, 0, af[0], bf[0]);
      __builtin_amdgcn_sched_barrier(0);
      mfma_slice(1);                                    // slice 3 lives in fragment set 1
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- KS > 1: add the groups' accumulators. Groups 1 .. KS-1 park theirs in LDS (the stages
  // are free now), register r of MFMA tile (i, j) of wavefront w at float index
  // ((w*TM*TN + i*TN + j)*16 + r)*64 + lane of the group's area (consecutive lanes, consecutive
  // words); group 0 adds them in the order 1, 2, ... and goes on to the epilogue alone.
  if (KS > 1) {
    static_assert(KS == 1 || (KS - 1) * BM * BN * 4 <= KS * Cfg::SMEM, "reduction area fits the stages");
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem_all);
    const int mine = wave * Cfg::TM * Cfg::TN * 16 * 64 + lane;
    if (kg > 0) {
      float* dst = red + (kg - 1) * (BM * BN) + mine;
#pragma unroll
      for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[((i * Cfg::TN + j) * 16 + r) * 64] = acc[i][j][r];
    }
    __syncthreads();
    if (kg > 0) return;
#pragma unroll
    for (int g2 = 1; g2 < KS; ++g2) {
      const float* src = red + (g2 - 1) * (BM * BN) + mine;
#pragma unroll
      for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] += src[((i * Cfg::TN + j) * 16 + r) * 64];
    }
  }

  // ---- epilogue: fp32 -> 16-bit (RNE), guarded element stores
  const int row_base = m0 + wm * (BM / WM) + 4 * (lane >> 5);
  const int col_base = n0 + wn * (BN / WN) + (lane & 31);
  // Plain 16-bit store with even N and ldc: neighbouring lanes (columns c, c+1 of the same rows)
  // exchange two of every four values, so that the even lane holds rows 0, 1 and the odd lane
  // rows 2, 3 of both columns of a register group: 32-bit stores, half as many.
  if (epi == 0 && bias == nullptr && !(N & 1) && !(ldc & 1) && !(reinterpret_cast<uintptr_t>(C) & 3)) {
    const bool odd = lane & 1;
    auto neighbour = [](float x) {                        // the value lane l ^ 1 passes in
      return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
    };
    const int col0 = col_base - (odd ? 1 : 0);
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
      for (int j = 0; j < Cfg::TN; ++j) {
        const int col = col0 + j * 32;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float got0 = neighbour(odd ? acc[i][j][4 * g] : acc[i][j][4 * g + 2]);
          const float got1 = neighbour(odd ? acc[i][j][4 * g + 1] : acc[i][j][4 * g + 3]);
          const uint32_t w0 = odd ? Elem<Tag>::pack2(got0, acc[i][j][4 * g + 2]) : Elem<Tag>::pack2(acc[i][j][4 * g], got0);
          const uint32_t w1 = odd ? Elem<Tag>::pack2(got1, acc[i][j][4 * g + 3]) : Elem<Tag>::pack2(acc[i][j][4 * g + 1], got1);
          const int row = row_base + i * 32 + 8 * g + (odd ? 2 : 0);
          if (col < N) {
            if (row < M) *reinterpret_cast<uint32_t*>(C + (int64_t)row * ldc + col) = w0;
            if (row + 1 < M) *reinterpret_cast<uint32_t*>(C + (int64_t)(row + 1) * ldc + col) = w1;
          }
        }
      }
    return;
  }
  gemm_epilogue<Tag>([&](auto&& out) {
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
      for (int j = 0; j < Cfg::TN; ++j) {
        const int col = col_base + j * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
          if (row < M && col < N) out((int64_t)row * ldc + col, col, acc[i][j][r]);
        }
      }
  }, C, epi, bias);
}

// ------------------------------------------------------------------------------------------
// General kernel: any M, N, K, leading dimensions and alignment. 64 x 64 x 32 tile, 4 wavefronts
// of 32 x 32, element-wise guarded loads with zero fill, B always staged as [n][k].
// ------------------------------------------------------------------------------------------
template <typename Tag>
__global__ __launch_bounds__(256) void gemm_general_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, int transB, uint16_t* __restrict__ C,
    int64_t ldc, int epi, const uint16_t* __restrict__ bias) {
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
      V8 a = lds_read8<V8>(reinterpret_cast<const char*>(As), ((wm * 32 + (lane & 31)) * LDS_S + off) * 2);
      V8 b = lds_read8<V8>(reinterpret_cast<const char*>(Bs), ((wn * 32 + (lane & 31)) * LDS_S + off) * 2);
      acc = mfma32(a, b, acc);
    }
    __syncthreads();
  }
  const int col = n0 + wn * 32 + (lane & 31);
  gemm_epilogue<Tag>([&](auto&& out) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < M && col < N) out((int64_t)row * ldc + col, col, acc[r]);
    }
  }, C, epi, bias);
}

// Second pass of a K split across workgroups: C = epilogue(sum over parts, in the order 0, 1, ...,
// of the fp32 partial products). One thread per four consecutive columns of a row.
template <typename Tag>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(
    int M, int N, int parts, const float* __restrict__ ws, int64_t part_stride,
    uint16_t* __restrict__ C, int64_t ldc, int epi, const uint16_t* __restrict__ bias) {
  const int nq = (N + 3) / 4;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)M * nq) return;
  const int row = (int)(t / nq), col0 = (int)(t % nq) * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const float* src = ws + (int64_t)row * N + col0;
  if (col0 + 3 < N && (N & 3) == 0) {
    for (int p = 0; p < parts; ++p) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(src + (int64_t)p * part_stride);
      acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
    }
  } else {
    for (int p = 0; p < parts; ++p)
      for (int e = 0; e < 4; ++e)
        if (col0 + e < N) acc[e] += src[(int64_t)p * part_stride + e];
  }
  gemm_epilogue<Tag>([&](auto&& out) {
    for (int e = 0; e < 4; ++e)
      if (col0 + e < N) out((int64_t)row * ldc + col0 + e, col0 + e, acc[e]);
  }, C, epi, bias);
}

// K == 0: the empty sum (only launched when C is overwritten; C += 0 is a no-op).
__global__ void gemm_zero_kernel(int M, int N, uint16_t* __restrict__ C, int64_t ldc) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < (int64_t)M * N) C[(e / N) * ldc + (e % N)] = 0;
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
template <typename Tag, int BM, int BN, int BK, int WM, int WN, bool TRANSB, int KS>
static int launch_tile(const GemmArgs& g, hipStream_t s) {
  typedef GemmTile<Tag, BM, BN, BK, WM, WN, TRANSB> Cfg;
  static_assert(Cfg::NT * KS <= 1024 && KS * Cfg::SMEM <= 160 * 1024, "one workgroup, one CU's LDS");
  auto kern = gemm_tile_kernel<Tag, BM, BN, BK, WM, WN, TRANSB, KS>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            KS * Cfg::SMEM) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nbm = (int)((g.M + BM - 1) / BM), nbn = (int)((g.N + BN - 1) / BN);
  if (g.parts <= 1) {
    hipLaunchKernelGGL(kern, dim3(nbm * nbn), dim3(Cfg::NT * KS), KS * Cfg::SMEM, s, (int)g.M, (int)g.N,
                       (int)g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc, nbm, nbn, device_xcds(), g.epi(), g.bias, 0,
                       (int64_t)0);
    return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
  }
  // K split across workgroups: fp32 partial tiles into the scratch, then the fixed-order sum
  const int KT = (int)((g.K + BK - 1) / BK);
  const int part_steps = (KT + g.parts - 1) / g.parts;
  const int parts = (KT + part_steps - 1) / part_steps;    // no empty part
  const int64_t part_stride = g.M * g.N;
  hipLaunchKernelGGL(kern, dim3(nbm * nbn, parts), dim3(Cfg::NT * KS), KS * Cfg::SMEM, s, (int)g.M,
                     (int)g.N, (int)g.K, g.A, g.lda, g.B, g.ldb, reinterpret_cast<uint16_t*>(g.scratch),
                     g.N, nbm, nbn, device_xcds(), (int)EPI_PART32, (const uint16_t*)nullptr, part_steps, part_stride);
  if (hipGetLastError() != hipSuccess) return MLT_ERR_LAUNCH;
  const int64_t nthreads = g.M * ((g.N + 3) / 4);
  hipLaunchKernelGGL(gemm_splitk_reduce_kernel<Tag>, dim3((unsigned)((nthreads + 255) / 256)), dim3(256),
                     0, s, (int)g.M, (int)g.N, parts, g.scratch, part_stride, g.C, g.ldc, g.epi(), g.bias);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

template <typename Tag>
static int launch_general(const GemmArgs& g, hipStream_t s) {
  dim3 grid((unsigned)((g.N + 63) / 64), (unsigned)((g.M + 63) / 64));
  hipLaunchKernelGGL(gemm_general_kernel<Tag>, grid, dim3(256), 0, s, (int)g.M, (int)g.N, (int)g.K,
                     g.A, g.lda, g.B, g.ldb, g.transB, g.C, g.ldc, g.epi(), g.bias);
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
  // K == 0: the empty sum; with a fused epilogue C = act(bias), which the general kernel's epilogue
  // computes after zero K steps
  if (g.K == 0 && !g.fused()) { p.variant = GEMM_ZERO; p.name = "gemm_zero"; return p; }
  if (g.K == 0 || !fast_path_ok(g) || g.forced == GEMM_GENERAL) {
    p.variant = GEMM_GENERAL; p.name = "gemm_general_64x64x32";
    p.bm = 64; p.bn = 64; p.bk = 32; p.wm = 2; p.wn = 2;
    return p;
  }
  // ---- the tile kernels: workgroup tile and K split
  // The candidate that needs the least time over the whole grid: (rounds of one workgroup per CU)
  // x (K steps of 64) x (its measured time per K step: two-group 256x256 kernel 1.17 us, older
  // 256x256 kernel 1.8 us; small tiles with the K steps split over 2 to 4 groups of wavefronts
  // inside the workgroup: 128x128 0.575 us, 64x128 0.37 us, 64x64 0.22 us; unsplit, for fewer than
  // 8 K steps: 0.60, 0.41, 0.35); ties go to the larger tile. (3072^3, 144 big tiles: 1033 TFLOP/s
  // against 739 with 576 tiles of 128x128; 2048^3, 64 big tiles: 437 against 758; 256 x 4096 x
  // 4096: 482 with 256 split tiles of 64x64, 326 unsplit, 244 with 64 tiles of 128x128.)
  // Never less than the time the operands take to arrive (A and B once at 5.2 TB/s: 64 x 8192 x
  // 28672 measured 91 us), more when too few workgroups pull or the last round leaves CUs idle
  // (the term is spelled out in the code below).
  // On top of that the K steps may be split over 2, 4 or 8 workgroups per tile (the small-tile
  // kernels), when the tiles alone leave most of the chip idle against a long K: each part writes
  // an fp32 partial tile to a scratch and a second kernel adds the parts in a fixed order
  // (deterministic; no atomics). Its price in the same units: a launch (4 us) plus writing and
  // reading parts * M * N floats at about 4 TB/s.
  DeviceInfo di;
  const int64_t NCU = device_info(di) && di.ncu > 0 ? di.ncu : 256;
  const int64_t KT = (g.K + 63) / 64;
  auto cost = [&](int64_t bm, int64_t bn, int64_t t_step, int64_t fixed, int parts, int kgroups) {
    const int64_t wgs = ((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn) * parts;
    const int64_t rounds = (wgs + NCU - 1) / NCU;
    const int64_t steps = (KT + parts - 1) / parts;
    const int64_t compute = rounds * (steps * t_step + fixed);
    // operand arrival: both operands once at 5.2 TB/s, which about 0.6 workgroups per CU already
    // draw (measured 37 GB/s per streaming workgroup: 64 of them 2.4 TB/s, 128 4.2, 224 5.7);
    // beyond one workgroup per CU the last round's idle CUs count (448 workgroups take the time
    // of 512: 32 x 28672 x 8192 measured 104-108 us on 64 x 64 tiles against 82 on 224 of 64 x 128)
    const int64_t base = (g.M + g.N) * g.K * 2 / 5200;
    // (the decode shapes are priced with B coming from memory: then fewer workgroups than CUs do
    // not keep enough bytes in flight; 64 x 8192 x 8192 on 128 tiles of 64 x 64: 43 us with B
    // rotating over more than the last-level cache holds, 34-37 us with K split two or four ways)
    const int64_t need = g.M <= 64 && g.transB ? NCU : 6 * NCU / 10;
    // B stored N x K: a workgroup reads (K groups) x 128 contiguous bytes of each row at a time.
    // The two-group tiles (256-byte pieces) need a workgroup on every CU and a little more to
    // draw the full rate (64 x 28672 x 8192 on 224 tiles of 64 x 128: 107 us = 1.18 x the 5.2 TB/s
    // time); the four-group 64 x 64 tile with between one and two workgroups per CU has them all
    // resident at once, so there is no second round with idle CUs (the same problem on 448 such
    // tiles: 102 us; 32 x 28672 x 8192: 95 against 105; 48 x ...: 95 against 100)
    const int64_t need_here = g.transB && kgroups == 2 && parts == 1 ? NCU + NCU / 20 : need;
    int64_t arrive = wgs >= NCU && wgs >= need_here ? base * rounds * NCU / wgs
                     : (wgs >= need_here ? base : base * need_here / wgs);
    if (g.transB && kgroups == 4 && parts == 1 && wgs > NCU && wgs <= 2 * NCU) arrive = base + base / 20;
    return (compute > arrive ? compute : arrive) + (parts > 1 ? 4000 + 2 * parts * g.M * g.N / 1000 : 0);
  };
  // Among the candidates within 8 % of the best estimate the largest tile wins (a larger tile
  // re-reads its operands from L2 less often, which the estimate leaves out: 64 x 8192 x 28672
  // measured 90 us on 64x128 tiles in four parts, 100-110 us on 64x64 tiles in two); for one tile
  // size, the fewer parts unless more parts are estimated more than 5 % faster.
  const bool pp = gemm_pp_ok(g);
  // t: ns per K step of 64; fixed: ns per round before the first and after the last step, where a
  // fit over K gave one (2048 x 2048 x K on the split 128 x 128 kernel: 0.56 us per step + 2 us)
  struct Cand { int variant; int bm, bn; int64_t t, fixed; int kgroups; };
  const Cand big = {pp ? GEMM_256_PP16 : GEMM_256_W8, 256, 256, pp ? 1170 : 1800, 0, 1};
  const Cand split[] = {{GEMM_128_K2, 128, 128, 560, 2000, 2}, {GEMM_64X128_K2, 64, 128, 370, 0, 2}, {GEMM_64_K4, 64, 64, 220, 0, 4}};
  const Cand whole[] = {{GEMM_128_W8, 128, 128, 600, 0, 1}, {GEMM_64X128_W8, 64, 128, 410, 0, 1}, {GEMM_64_W4, 64, 64, 350, 0, 1}};
  struct Choice { int variant, parts, area; int64_t t; };
  Choice all[20];
  int n_all = 0;
  // no tile taller or wider than the matrix rounded up to 64 (it would multiply padding)
  auto fits = [&](int bm, int bn) {
    return !(bm > 64 && bm > (g.M + 63) / 64 * 64) && !(bn > 64 && bn > (g.N + 63) / 64 * 64);
  };
  if (g.forced_parts <= 1 && fits(256, 256)) all[n_all++] = Choice{big.variant, 1, 256 * 256, cost(256, 256, big.t, 0, 1, 1)};
  // The two-group kernel on 128 x 128 tiles, no K split across workgroups, in its two forms (fits
  // over K at 256 and 512 tiles, kernel time without the call):
  //   K steps of 64, two workgroups per CU: 0.84 us per step for a pair of tiles + 1.9 us per pair,
  //     0.52 us + 4 us for a tile alone on its CU;
  //   K steps of 128, one workgroup per CU: 0.436 us per 64 of K + 4.3 us per round.
  // One tile per CU: the 128-deep form (1024 x 4096 x 4096: 35.4 us against 40.8 on the register-
  // staged split kernel and 43.3 on the 64-deep form, hipBLASLt 36.6; 2048^3: 22.9 against 25.5,
  // hipBLASLt 25.3; 512 x 8192 x 8192: 65.7 against 76.4, hipBLASLt 64.1). Two tiles per CU: the
  // 64-deep form, whose workgroups hide each other's start and end (2048 x 4096 x 4096: 60.0
  // against 69.6 us, 82 on the split kernel, 73 on 128 big tiles; 1024 x 8192 x 8192: 114 against
  // 132, 153 and 134).
  if (pp && g.forced_parts <= 1 && fits(128, 128)) {
    const int64_t wgs = ((g.M + 127) / 128) * ((g.N + 127) / 128);
    const int64_t base = (g.M + g.N) * g.K * 2 / 5200;
    const int64_t need = 6 * NCU / 10;
    const int64_t arrive = wgs >= need ? base : base * need / wgs;
    const int64_t pairs = wgs / (2 * NCU), rem = wgs - pairs * 2 * NCU;
    const int64_t own64 = pairs * (KT * 840 + 1900) +
                          (rem > NCU ? KT * 840 + 1900 : rem > 0 ? KT * 519 + 4000 : 0);
    // (with at most one tile per CU and K a multiple of 128 the 128-deep form is never slower, also
    // where both are bound by operand arrival: 128 x 28672 x 8192 116 against 134 us)
    if (wgs > NCU || g.K % 128 != 0)
      all[n_all++] = Choice{GEMM_128_PP16, 1, 128 * 128, own64 > arrive ? own64 : arrive};
    if (g.K % 128 == 0) {
      const int64_t own128 = ((wgs + NCU - 1) / NCU) * (KT * 436 + 4300);
      all[n_all++] = Choice{GEMM_128_PP16_K128, 1, 128 * 128, own128 > arrive ? own128 : arrive};
    }
  }
  for (int parts = g.forced_parts > 0 ? g.forced_parts : 1; parts <= (g.forced_parts > 0 ? g.forced_parts : 8); parts *= 2) {
    // every part keeps at least 8 K steps, and its partial tiles must fit the scratch allowed
    if (parts > 1 && KT < 8 * parts) break;
    if (parts > 1 && g.scratch_limit >= 0 && (int64_t)parts * g.M * g.N * 4 > g.scratch_limit) break;
    for (const auto& c : KT / parts >= 8 ? split : whole) {
      if (!fits(c.bm, c.bn)) continue;
      all[n_all++] = Choice{c.variant, parts, c.bm * c.bn, cost(c.bm, c.bn, c.t, c.fixed, parts, c.kgroups)};
    }
  }
  if (n_all == 0) all[n_all++] = Choice{big.variant, 1, 256 * 256, cost(256, 256, big.t, 0, 1, 1)};
  int64_t best = all[0].t;
  for (int i = 1; i < n_all; ++i) best = all[i].t < best ? all[i].t : best;
  Choice pick = all[0];
  bool have = false;
  for (int i = 0; i < n_all; ++i) {
    if (all[i].t > best + best / 12) continue;
    bool better = !have || all[i].area > pick.area;
    if (have && all[i].area == pick.area) {
      // same tile: the fewer parts, unless more parts are estimated more than 5 % faster
      if (all[i].parts == pick.parts) better = all[i].t < pick.t;
      else if (all[i].parts < pick.parts) better = all[i].t <= pick.t + pick.t / 20;
      else better = all[i].t + all[i].t / 20 < pick.t;
    }
    if (better) pick = all[i];
    have = true;
  }
  int v = pick.variant;
  const int best_parts = pick.parts;
  // ---- the skinny kernels (B stored N x K, no LDS staging of A): the automatic choice for one
  // 16-row tile of A, and for two when they beat the tile kernels' estimate; B streamed through
  // an LDS ring (16 columns x 512 k per stage, the A fragments of a k stage shared by a group of
  // column blocks) once B is well beyond the caches: measured 5.7 TB/s of B for M <= 16; for two
  // row tiles 4.7-5.9 TB/s with 16384 columns or more and 3.0-4.6 TB/s with fewer (32 x 8192 x
  // 28672: 103 us, against 85 us for the tile kernels with K split four ways). The rates that
  // decide are those with B coming from memory, as the weights of a decoder do (every matrix is
  // read once per token, and a model is far larger than the 256 MiB last-level cache): the
  // streaming kernel's non-temporal loads make it indifferent to what that cache holds, while the
  // tile kernels run up to 40 % faster when the same B of less than 256 MB is multiplied again
  // and again (32 x 16384 x 8192: tile kernels 41 us on a repeated B and 59 us on rotating ones,
  // the streaming kernel 55 and 56 us; 32 x 65536 x 2048: 43 / 65 against 53 / 54 us). Taller A
  // goes to the tile kernels, which stage A through LDS once per tile (64 x 28672 x 8192: 99 us
  // against 160 us streaming; 64 x 14336 x 4096: 20 us against 43 us).
  const bool big_b = g.N * g.K >= ((int64_t)1 << 25);
  const int64_t two_tile_rate = g.N >= 16384 ? 5600 : 3900;  // bytes of B per us, B from memory
  const bool stream_wins = g.M <= 16 || g.N * g.K * 2 / two_tile_rate < best;
  const bool skinny_auto = g.forced == GEMM_AUTO && g.M <= 32 && (!big_b || stream_wins);
  if ((g.forced == GEMM_SKINNY_DMA || (skinny_auto && big_b)) && gemm_skinny_dma_ok(g)) {
    p.variant = GEMM_SKINNY_DMA;
    p.name = "gemm_nt_skinny_16cols_stream";
    p.bm = (int)((g.M + 15) / 16) * 16; p.bn = 16; p.bk = 512;
    p.wm = 1; p.wn = 1;
    p.mfma_m = 16; p.mfma_n = 16; p.mfma_k = 32;
    return p;
  }
  if ((skinny_auto || g.forced == GEMM_SKINNY || g.forced == GEMM_SKINNY_DMA) && gemm_skinny_ok(g)) {
    p.variant = GEMM_SKINNY; p.name = "gemm_nt_skinny_16cols_ksplit8";
    p.bm = (int)((g.M + 15) / 16) * 16; p.bn = 16; p.bk = 32; p.wm = 1; p.wn = 1;
    p.mfma_m = 16; p.mfma_n = 16; p.mfma_k = 32;
    return p;
  }
  if (g.forced >= GEMM_256 && g.forced < GEMM_NUM_VARIANTS && g.forced != GEMM_SKINNY &&
      g.forced != GEMM_SKINNY_DMA)
    v = g.forced;
  if ((v == GEMM_256_PP16 || v == GEMM_256_W4) && !gemm_pp_ok(g)) v = GEMM_256_W8;
  if (v == GEMM_128_PP16_K128 && (!gemm_pp_ok(g) || g.K % 128)) v = GEMM_128_PP16;
  if (v == GEMM_128_PP16 && !gemm_pp_ok(g)) v = GEMM_128_W8;
  // a forced kernel keeps the split only if it is one of the kernels that can run it
  const bool can_split = v == GEMM_128_K2 || v == GEMM_64X128_K2 || v == GEMM_64_K4 || v == GEMM_128_W8 ||
                         v == GEMM_64X128_W8 || v == GEMM_64_W4;
  p.parts = can_split ? best_parts : 1;
  p.scratch_bytes = p.parts > 1 ? (int64_t)p.parts * g.M * g.N * 4 : 0;
  p.variant = v;
  p.bk = 64;
  switch (v) {
    case GEMM_256: p.bm = p.bn = 256; p.wm = 2; p.wn = 2;
      p.name = g.transB ? "gemm_nt_256x256x64_w2x2" : "gemm_nn_256x256x64_w2x2"; break;
    case GEMM_256_W8: p.bm = p.bn = 256; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_256x256x64_w2x4" : "gemm_nn_256x256x64_w2x4"; break;
    case GEMM_256_W8X1: p.bm = p.bn = 256; p.wm = 8; p.wn = 1;
      p.name = g.transB ? "gemm_nt_256x256x64_w8x1" : "gemm_nn_256x256x64_w8x1"; break;
    case GEMM_256_W1X8: p.bm = p.bn = 256; p.wm = 1; p.wn = 8;
      p.name = g.transB ? "gemm_nt_256x256x64_w1x8" : "gemm_nn_256x256x64_w1x8"; break;
    case GEMM_256_PP16: p.bm = p.bn = 256; p.wm = 2; p.wn = 4;
      p.mfma_m = 16; p.mfma_n = 16; p.mfma_k = 32;
      p.name = g.transB ? "gemm_nt_256x256x64_w2x4_pp16" : "gemm_nn_256x256x64_w2x4_pp16"; break;
    case GEMM_128_PP16: p.bm = p.bn = 128; p.wm = 2; p.wn = 4;
      p.mfma_m = 16; p.mfma_n = 16; p.mfma_k = 32;
      p.name = g.transB ? "gemm_nt_128x128x64_w2x4_pp16" : "gemm_nn_128x128x64_w2x4_pp16"; break;
    case GEMM_128_PP16_K128: p.bm = p.bn = 128; p.bk = 128; p.wm = 2; p.wn = 4;
      p.mfma_m = 16; p.mfma_n = 16; p.mfma_k = 32;
      p.name = g.transB ? "gemm_nt_128x128x128_w2x4_pp16" : "gemm_nn_128x128x128_w2x4_pp16"; break;
    case GEMM_256_W4: p.bm = p.bn = 256; p.wm = 2; p.wn = 2;
      p.name = g.transB ? "gemm_nt_256x256x64_w2x2_swp" : "gemm_nn_256x256x64_w2x2_swp"; break;
    case GEMM_128_W8: p.bm = p.bn = 128; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_128x128x64_w2x4" : "gemm_nn_128x128x64_w2x4"; break;
    case GEMM_64X128_W8: p.bm = 64; p.bn = 128; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_64x128x64_w2x4" : "gemm_nn_64x128x64_w2x4"; break;
    case GEMM_64_W4: p.bm = p.bn = 64; p.wm = 2; p.wn = 2;
      p.name = g.transB ? "gemm_nt_64x64x64_w2x2" : "gemm_nn_64x64x64_w2x2"; break;
    case GEMM_128_K2: p.bm = p.bn = 128; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_128x128x64_w2x4_k2" : "gemm_nn_128x128x64_w2x4_k2"; break;
    case GEMM_64X128_K2: p.bm = 64; p.bn = 128; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_64x128x64_w2x4_k2" : "gemm_nn_64x128x64_w2x4_k2"; break;
    case GEMM_64_K4: p.bm = p.bn = 64; p.wm = 2; p.wn = 2;
      p.name = g.transB ? "gemm_nt_64x64x64_w2x2_k4" : "gemm_nn_64x64x64_w2x2_k4"; break;
    default: p.variant = GEMM_256_W8; p.bm = p.bn = 256; p.wm = 2; p.wn = 4;
      p.name = g.transB ? "gemm_nt_256x256x64_w2x4" : "gemm_nn_256x256x64_w2x4"; break;
  }
  return p;
}

// KS: K-split groups per workgroup when B is stored N x K, KS_NN when it is stored K x N (whose
// padded stage is larger, so fewer groups fit the LDS).
template <typename Tag, int BM, int BN, int BK, int WM, int WN, int KS = 1, int KS_NN = KS>
static int launch_tile_tb(const GemmArgs& g, hipStream_t s) {
  return g.transB ? launch_tile<Tag, BM, BN, BK, WM, WN, true, KS>(g, s)
                  : launch_tile<Tag, BM, BN, BK, WM, WN, false, KS_NN>(g, s);
}

template <typename Tag>
static int run_gemm_t(const GemmArgs& g, const GemmPlan& p, hipStream_t s) {
  switch (p.variant) {
    case GEMM_ZERO: {
      if (g.acc32) return MLT_OK;
      const int64_t n = g.M * g.N;
      hipLaunchKernelGGL(gemm_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                         (int)g.M, (int)g.N, g.C, g.ldc);
      return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
    }
    case GEMM_GENERAL: return launch_general<Tag>(g, s);
    case GEMM_256: return launch_tile_tb<Tag, 256, 256, 64, 2, 2>(g, s);
    case GEMM_256_W8: return launch_tile_tb<Tag, 256, 256, 64, 2, 4>(g, s);
    case GEMM_256_W8X1: return launch_tile_tb<Tag, 256, 256, 64, 8, 1>(g, s);
    case GEMM_256_W1X8: return launch_tile_tb<Tag, 256, 256, 64, 1, 8>(g, s);
    case GEMM_128_W8: return launch_tile_tb<Tag, 128, 128, 64, 2, 4>(g, s);
    case GEMM_64X128_W8: return launch_tile_tb<Tag, 64, 128, 64, 2, 4>(g, s);
    case GEMM_64_W4: return launch_tile_tb<Tag, 64, 64, 64, 2, 2>(g, s);
    case GEMM_128_K2: return launch_tile_tb<Tag, 128, 128, 64, 2, 4, 2>(g, s);
    case GEMM_64X128_K2: return launch_tile_tb<Tag, 64, 128, 64, 2, 4, 2>(g, s);
    case GEMM_64_K4: return launch_tile_tb<Tag, 64, 64, 64, 2, 2, 4, 3>(g, s);
    case GEMM_256_PP16: return run_gemm_pp(g, 256, 64, s);
    case GEMM_128_PP16: return run_gemm_pp(g, 128, 64, s);
    case GEMM_128_PP16_K128: return run_gemm_pp(g, 128, 128, s);
    case GEMM_256_W4: return run_gemm_w4(g, s);
    case GEMM_SKINNY: return run_gemm_skinny(g, s);
    case GEMM_SKINNY_DMA: return run_gemm_skinny_dma(g, s);
  }
  return MLT_ERR_UNSUPPORTED;
}

// Scratch for the partial products of a K split across workgroups: one buffer per (device, stream)
// pair, so that calls on different streams never share one; allocated at the first call that needs
// it (hipMalloc; no device synchronisation), grown by doubling (the smaller buffer is kept until the
// process ends: work already enqueued may still use it), used in stream order. The table is
// small and fixed; when it is full, or an allocation fails, the call gets a stream-ordered
// allocation of its own (or, if that fails too, runs without the split).
namespace {
struct ScratchSlot { int dev; hipStream_t stream; float* ptr; int64_t bytes; };
constexpr int kScratchSlots = 32;
ScratchSlot g_scratch[kScratchSlots];
int g_scratch_used = 0;
std::mutex g_scratch_mu;

}  // namespace

// true while `s` records into a graph: nothing may be allocated then
static bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
  return st != hipStreamCaptureStatusNone;
}

float* cached_scratch(int64_t bytes, hipStream_t s) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  ScratchSlot* slot = nullptr;
  for (int i = 0; i < g_scratch_used; ++i)
    if (g_scratch[i].dev == dev && g_scratch[i].stream == s) slot = &g_scratch[i];
  if (slot && slot->bytes >= bytes) return slot->ptr;
  if (!slot) {
    if (g_scratch_used == kScratchSlots) return nullptr;
    slot = &g_scratch[g_scratch_used];
    *slot = ScratchSlot{dev, s, nullptr, 0};
  }
  // a buffer that is there is used under capture as well; a new one is not allocated in the
  // middle of a capture (the call then runs without the split; mlt_gemm_noalloc is the entry point
  // made for captured code)
  if (stream_is_capturing(s)) return nullptr;
  int64_t want = slot->bytes > 0 ? 2 * slot->bytes : (int64_t)4 << 20;
  while (want < bytes) want *= 2;
  void* p = nullptr;
  if (hipMalloc(&p, (size_t)want) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
  if (slot == &g_scratch[g_scratch_used]) ++g_scratch_used;
  slot->ptr = static_cast<float*>(p);
  slot->bytes = want;
  return slot->ptr;
}

// The scratch of the entry point that may not allocate (mlt_gemm_noalloc): a fixed array in
// device memory, one copy per GPU the library runs on, held until the process ends. In host code
// the array's name is only a handle; its device address is looked up once per device, with that
// device current, and only that address is ever handed to kernels. Every call on a GPU shares
// that GPU's array (calls that overlap on one GPU race); nothing in it has to start at zero: each
// part of a K split writes every element of its slice before the second kernel reads them.
namespace {
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];
constexpr int kMaxDevices = 64;
float* g_static_scratch[kMaxDevices];
std::mutex g_static_scratch_mu;
}  // namespace

float* static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  std::lock_guard<std::mutex> lock(g_static_scratch_mu);
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
    g_static_scratch[dev] = static_cast<float*>(p);
  }
  return g_static_scratch[dev];
}

int run_gemm(const GemmArgs& g_in, GemmPlan& p, hipStream_t s) {
  GemmArgs g = g_in;
  g.parts = p.parts;
  bool own = false;
  if (p.parts > 1 && !g.scratch) {
    g.scratch = cached_scratch(p.scratch_bytes, s);
    if (!g.scratch) {
      void* ws = nullptr;
      if (!stream_is_capturing(s) && hipMallocAsync(&ws, (size_t)p.scratch_bytes, s) == hipSuccess && ws) {
        g.scratch = static_cast<float*>(ws);
        own = true;
      } else {
        (void)hipGetLastError();
        g.parts = 1;
        p.parts = 1;                                       // what ran, for the reported kernel name
        p.scratch_bytes = 0;
      }
    }
  }
  const int rc = g.dtype == MLT_BF16 ? run_gemm_t<bf16_tag>(g, p, s) : run_gemm_t<f16_tag>(g, p, s);
  if (own) (void)hipFreeAsync(g.scratch, s);
  return rc;
}

}  // namespace mlt
