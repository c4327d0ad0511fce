// GEMM C = A*B for gfx950, two-group ("ping-pong") schedule with direct global->LDS loads.
//
// Same three levels as the paper's GEMM (arXiv 2503.14985, Sections 2.1-2.3: workgroup tile,
// per-warp sub-tile, hardware dot): workgroup tile 256 x 256, K step 64, 8 wavefronts as 2 x 4
// owning 128 x 64 each, MFMA 16x16x32 (MS = 16, the form the library uses) or 32x32x16 (MS = 32).
// What differs from gemm.hip is how memory traffic and
// matrix work overlap. A CU runs one workgroup, two wavefronts per SIMD. The two wavefronts of a
// SIMD are kept half a K step apart by one extra barrier at the start: while one of them issues
// its 64 (or 32) MFMAs of a K step back to back (compute phase), the other refills its operand fragments
// from LDS for its next compute phase (memory phase). Every phase ends in a workgroup barrier, so
// the matrix pipe of each SIMD always has exactly one wavefront feeding it and LDS latency never
// sits in front of an MFMA.
//
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l of a
// wavefront writes 16 bytes at base + 16*l). LDS (160 KB) is a ring of five 32 KB slots holding
// the sequence A_0 B_0 A_1 B_1 A_2 ... (A_k, B_k: the operand tiles of K step k), i.e. two and a
// half K steps. That extra half step is what lets every load be issued from a memory phase: the
// vector memory path of a CU moves 64 bytes per clock, so the 64 KB of a K step occupy it for
// half of the 2048 clocks the MFMAs of that step take, and a wavefront that issues loads in
// front of its MFMAs stalls the matrix pipe. Group 1 fetches the A tiles, group 0 the B tiles.
// Because the LDS side of such a
// load is contiguous per wavefront, the tiles are stored unpadded and bank conflicts are avoided
// by choosing WHICH 16-byte chunk of global memory each lane fetches (an XOR swizzle):
//   A tile  [256 rows][8 chunks of 8 k]   chunk c of row r sits in slot c ^ ((r >> 1) & 7)
//   B tile, B given as N x K: same as A with n as the row
//   B tile, B given as K x N: [64 k][32 chunks of 8 n], chunk q of row k sits in slot q ^ 4*(k & 3)
//                             (16x16x32 form: q ^ (4*(k & 3) + 2*((k >> 3) & 1)), see swz_kn)
// With these, the 16 lanes that the LDS serves together hit 16 distinct 16-byte bank groups, for
// the row reads (ds_read_b128) and for the transposing reads (ds_read_b64_tr_b16) alike.
//
// Requirements (checked by the host): K % 64 == 0, lda % 8 == 0, ldb % 8 == 0, N % 8 == 0 when B
// is K x N, A and B 16-byte aligned, 256 * lda and 64 * ldb + N below 2^30 elements (32-bit
// per-lane byte offsets). M and N need not be multiples of 256: out-of-range rows/columns are
// clamped on load and never stored.
#include <type_traits>

#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

constexpr int PP_NT = 512;
constexpr int PP_NSLOT = 5;
// The workgroup tile is BT x BT (BT = 256: one workgroup per CU, the 160 KB ring described above;
// BT = 128: the same schedule with 64 x 32 per wavefront, 16 KB slots and at most 128 registers,
// so that two workgroups share a CU and one computes while the other waits at a barrier).
// BK is the K step: 64, or 128 for BT = 128 (32 KB slots again, one workgroup per CU, phases of
// twice the length: with 64 x 32 per wavefront a compute phase of one 64-deep step is only 256
// clocks of MFMA, and the fixed cost of a phase change then costs as much as the phase).
template <int BT, int BK> struct PpTile {
  static constexpr int SLOT = BT * BK * 2;               // one operand tile
  static constexpr int SMEM = PP_NSLOT * SLOT;
  static constexpr int NL = SLOT / 1024 / 4;             // 1 KB blocks per wavefront and tile
  static constexpr int AROW = BK * 2;                    // bytes per row of the A (or N x K) tile
  static constexpr int CPR = BK / 8;                     // 16-byte k chunks per row: 8 or 16
  // chunk c of row r sits in slot c ^ swz(r): 16 consecutive rows at one chunk must fall in 16
  // distinct 16-byte bank groups of the 256-byte bank cycle
  static __device__ __forceinline__ int swz(int r) { return BK == 64 ? (r >> 1) & 7 : r & 15; }
};

// Workgroup id -> C tile: bands of 4 tile rows, column by column, so an XCD's 32 resident
// workgroups form a 4 x 8 block of tiles that shares 4 row panels of A and 8 column panels of B.
// (Measured at 8192^3: bands of 4 rows 0.8 % faster than bands of 8 with B stored K x N, 2.4 % with
// B stored N x K; 2, 5, 6 rows slower, 32 rows -5 %.)
constexpr int PP_GROUP_M = 4;

// Swizzle of the K x N operand tile ([64 k][32 chunks of 8 n]): chunk q of row k sits in slot
// q ^ swz_kn(k). A transposing read serves 32 lanes at a time (8 bytes each). With 32-wide tiles
// those are two 16-lane groups on the SAME four k rows and different chunks, and 4*(k & 3)
// separates the rows; with 16-wide tiles they are two groups on k rows 8 apart, which in addition
// need the 2*((k >> 3) & 1) term to land in different banks.
template <int MS>
__device__ __forceinline__ int swz_kn(int k) {
  return MS == 32 ? 4 * (k & 3) : 4 * (k & 3) + 2 * ((k >> 3) & 1);
}

template <int MS, typename V8>
__device__ __forceinline__ auto mfma_ms(V8 a, V8 b, typename std::conditional<MS == 32, f32x16, f32x4>::type c) {
  if constexpr (MS == 32) return mfma32(a, b, c);
  else return mfma16(a, b, c);
}

}  // namespace

template <typename Tag, bool TRANSB, int MS, int BT, int BK>
__global__ __launch_bounds__(PP_NT, (BT == 128 && BK == 64) ? 4 : 1) void gemm_pp_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc, int nbm,
    int nbn, int nxcd, int epi, const uint16_t* __restrict__ bias) {
  typedef typename Elem<Tag>::vec8 V8;
  typedef PpTile<BT, BK> T;
  static_assert((BT == 256 && BK == 64) || (BT == 128 && MS == 16 && (BK == 64 || BK == 128)),
                "tile sizes that were built and measured");
  constexpr int PP_BM = BT, PP_BN = BT, PP_SLOT = T::SLOT, NL = T::NL, PP_BK = BK;
  constexpr int AROW = T::AROW, CPR = T::CPR, RPBA = 64 / CPR;   // A tile: row bytes, chunks per row, rows per 1 KB block
  constexpr int WTM = BT / 2, WTN = BT / 4;              // per wavefront: 128 x 64 / 64 x 32
  constexpr int BROW = BT * 2;                           // bytes per k row of the K x N tile
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;               // 2 x 4 wavefronts
  const int grp = wm;                                    // waves 0-3 / 4-7: one of each per SIMD
  int tile_m, tile_n;
  tile_of_block<PP_GROUP_M>(blockIdx.x, nbm, nbn, nxcd, tile_m, tile_n);
  const int m0 = tile_m * PP_BM, n0 = tile_n * PP_BN;

  // ---- global -> LDS assignments. A tile is 32 (16) blocks of 1 KB (64 lanes x 16 bytes). The
  // four wavefronts of group 1 fill the A tiles, those of group 0 the B tiles, NL blocks each;
  // lane l owns the 16-byte slot l of a block.
  const char* ld_base;                                   // uniform: tile origin at k = 0
  int64_t ld_kstep;                                      // uniform: bytes per K step
  uint32_t voff[NL];
  if (grp == 1) {
    ld_base = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    ld_kstep = PP_BK * 2;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = ((wave & 3) * NL + i) * RPBA + lane / CPR;  // tile row held by this slot
      const int c = (lane % CPR) ^ T::swz(r);                   // k chunk stored in this slot
      const int rr = (m0 + r < M) ? r : (M - 1 - m0);
      voff[i] = (uint32_t)rr * (uint32_t)lda * 2u + (uint32_t)c * 16u;
    }
  } else if (TRANSB) {
    ld_base = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
    ld_kstep = PP_BK * 2;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = ((wave & 3) * NL + i) * RPBA + lane / CPR;
      const int c = (lane % CPR) ^ T::swz(r);
      const int rr = (n0 + r < N) ? r : (N - 1 - n0);
      voff[i] = (uint32_t)rr * (uint32_t)ldb * 2u + (uint32_t)c * 16u;
    }
  } else {
    ld_base = reinterpret_cast<const char*>(B);
    ld_kstep = (int64_t)PP_BK * ldb * 2;
    constexpr int LPR = BT / 8, RPB = 64 / LPR;             // lanes per k row, k rows per block
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int k = ((wave & 3) * NL + i) * RPB + lane / LPR;  // tile k row held by this slot
      const int q = (lane % LPR) ^ swz_kn<MS>(k);              // n chunk stored in this slot
      const int col = n0 + q * 8;
      voff[i] = (uint32_t)k * (uint32_t)ldb * 2u + (uint32_t)(col < N ? col : 0) * 2u;
    }
  }
  const int KT = K / PP_BK;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;      // LDS byte address of the buffer
  // this wavefront's NL blocks of operand tile t (A_t for group 1, B_t for group 0) into a slot
  // (an operand that only one row or column of tiles reads is read exactly once: streaming form)
  const bool stream = grp == 1 ? nbn == 1 : nbm == 1;
  auto issue_loads = [&](int t, int slot) {
    const char* gp = ld_base + (int64_t)t * ld_kstep;
    const uint32_t dst = lds0 + slot * PP_SLOT + (wave & 3) * (NL * 1024);
    if (stream) {
#pragma unroll
      for (int i = 0; i < NL; ++i) load_lds16_stream(gp, voff[i], dst + i * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) load_lds16(gp, voff[i], dst + i * 1024);
    }
  };
  // ---- fragment addresses inside a stage (per lane; tile and k slice offsets are immediates)
  // MS = 32: MFMA 32x32x16, 4 k slices of 16 per K step, A tiles of 32 rows, B tiles of 32 columns.
  // MS = 16: MFMA 16x16x32, 2 k slices of 32, tiles of 16. Both read the same bytes from LDS per
  // flop (a fragment is 1 KB either way); the 16x16x32 form updates half as many accumulator
  // registers per flop, and measured on N(0,1) operands the chip sustains 2100 TFLOP/s of it
  // against 1850 TFLOP/s of 32x32x16 (a register-only MFMA loop; power-limited clocks 2.05 against
  // 1.81 GHz).
  constexpr int NS = BK / (MS == 32 ? 16 : 32);           // k slices per K step
  constexpr int TA = WTM / MS, TB = WTN / MS;             // A / B tiles per wavefront
  const int lq = lane & (MS - 1), h = lane / MS;          // row (column) within a tile, k chunk of the slice
  constexpr int CPS = 64 / MS;                            // 16-byte k chunks per slice (2 or 4)
  int a_off[NS], b_off[4];
  {
    const int r = wm * WTM + lq;
    const int f = T::swz(lq);
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) a_off[kk] = r * AROW + (((CPS * kk + h) ^ f) * 16);
  }
  if (TRANSB) {
    const int r = wn * WTN + lq;
    const int f = T::swz(lq);
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) b_off[kk] = r * AROW + (((CPS * kk + h) ^ f) * 16);
  } else if (MS == 32) {
    // transposing read: 16-lane group g serves columns 16*(g%2).. of the 32-wide tile and k slots
    // 8*(g/2)..; lane s of the group addresses k row s/4 (+4 for the second read), columns 4*(s%4)..
    const int g = lane >> 4, s = lane & 15;
    const int krow = 8 * (g >> 1) + (s >> 2);
    const int q = wn * 8 + 2 * (g & 1) + ((s & 3) >> 1);
    const int x = 4 * (s >> 2);
    b_off[0] = krow * BROW + ((q ^ x) * 16) + 8 * (s & 1);        // column tile 0
    b_off[1] = krow * BROW + (((q + 4) ^ x) * 16) + 8 * (s & 1);  // column tile 1
    b_off[2] = b_off[3] = 0;
  } else {
    // 16-wide tiles: 16-lane group g serves k slots 8*g.. of the 32-deep slice for all 16 columns;
    // lane s addresses k row s/4 (+4 for the second read), columns 4*(s%4)..
    const int g = lane >> 4, s = lane & 15;
    const int krow = 8 * g + (s >> 2);
    const int x = swz_kn<16>(krow);
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int q = wn * (WTN / 8) + 2 * j + ((s & 3) >> 1);
      b_off[j] = krow * BROW + ((q ^ x) * 16) + 8 * (s & 1);
    }
  }

  typedef typename std::conditional<MS == 32, f32x16, f32x4>::type AccT;
  AccT acc[TA][TB];
#pragma unroll
  for (int i = 0; i < TA; ++i)
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int r = 0; r < (MS == 32 ? 16 : 4); ++r) acc[i][j][r] = 0.f;

  V8 af[NS][TA], bf[NS][TB];                              // [k slice][tile]
  auto read_frags = [&](const char* sa, const char* sb) {
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) {
#pragma unroll
      for (int i = 0; i < TA; ++i) af[kk][i] = lds_read8<V8>(sa, a_off[kk] + i * MS * AROW);
#pragma unroll
      for (int j = 0; j < TB; ++j) {
        if (TRANSB) {
          bf[kk][j] = lds_read8<V8>(sb, b_off[kk] + j * MS * AROW);
        } else {
          const int o = b_off[j] + kk * (BK / NS) * BROW;
          const s16x4 lo = lds_read_tr4(sb, o);
          const s16x4 hi = lds_read_tr4(sb, o + 4 * BROW);
          bf[kk][j] = join_tr<V8>(lo, hi);
        }
      }
    }
  };


  // Phase p ends at workgroup barrier p. Group 0 reads tile k (A_k and B_k) in phase 2k and
  // multiplies in phase 2k+1; group 1 does the same one phase later. Operand tile number h
  // (A_k: h = 2k, B_k: h = 2k+1) lives in slot h % 5 and is last read in phase 2k+1.
  //   group 1, memory phase of step k (phase 2k+1): issues A_{k+2} into the slot B_{k-1} left in
  //     phase 2k-1, then makes sure A_{k+1} (issued one step earlier) has landed: at most the NL
  //     loads just issued may still be in flight;
  //   group 0, memory phase of step k (phase 2k): issues B_{k+1} into the slot A_{k-1} left in
  //     phase 2k-1, and waits for it at the end of its compute phase (phase 2k+1).
  // Either way tile k+1 is complete when barrier 2k+1 releases, and its first reader (group 0,
  // phase 2k+2) comes after that barrier.
  if (grp == 1) {
    issue_loads(0, 0);
    if (KT > 1) { issue_loads(1, 2); __builtin_amdgcn_s_waitcnt(wait_imm(NL, 15)); }
    else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
  } else {
    issue_loads(0, 1);
    if (KT > 1) { issue_loads(1, 3); __builtin_amdgcn_s_waitcnt(wait_imm(NL, 15)); }
    else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
  }
  MLT_BARRIER();
  if (grp == 1) MLT_BARRIER();

  int slot_a = 0;                                         // slot of A_k; B_k is in the next one
  for (int k = 0; k < KT; ++k) {
    const int slot_b = slot_a + 1 == PP_NSLOT ? 0 : slot_a + 1;
    // ---- memory phase
    read_frags(smem + slot_a * PP_SLOT, smem + slot_b * PP_SLOT);
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 1) {
      if (k + 2 < KT) {
        issue_loads(k + 2, slot_a + 4 >= PP_NSLOT ? slot_a + 4 - PP_NSLOT : slot_a + 4);
        __builtin_amdgcn_s_waitcnt(wait_imm(NL, 0));
      } else {
        __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
      }
    } else {
      if (k >= 1 && k + 1 < KT)
        issue_loads(k + 1, slot_a + 3 >= PP_NSLOT ? slot_a + 3 - PP_NSLOT : slot_a + 3);
      __builtin_amdgcn_s_waitcnt(wait_imm(63, 0));
    }
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    // ---- compute phase
#pragma unroll
    for (int kk = 0; kk < NS; ++kk)
#pragma unroll
      for (int i = 0; i < TA; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j) acc[i][j] = mfma_ms<MS>(af[kk][i], bf[kk][j], acc[i][j]);
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 0) __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    slot_a = slot_a + 2 >= PP_NSLOT ? slot_a + 2 - PP_NSLOT : slot_a + 2;
  }
  if (grp == 0) MLT_BARRIER();

  // ---- epilogue: fp32 -> 16-bit (RNE) and store, or add to the fp32 C; guarded per element
  // accumulator register r of a 32x32 tile is row 8*(r/4) + 4*(l/32) + r%4, of a 16x16 tile row
  // 4*(l/16) + r; the column is the lane's
  const int row_base = m0 + wm * WTM + 4 * h;
  const int col_base = n0 + wn * WTN + lq;
  if constexpr (MS == 16) {
    // Plain 16-bit store with even N and ldc: neighbouring lanes (columns c, c+1 of the same four
    // rows) exchange two of their four values, so that the even lane holds rows 0, 1 and the odd
    // lane rows 2, 3 of BOTH columns: two 32-bit stores per tile and lane instead of four 16-bit
    // ones (the stores are what the epilogue spends its time on).
    const bool pairs = epi == 0 && bias == nullptr && !(N & 1) && !(ldc & 1) &&
                       !(reinterpret_cast<uintptr_t>(C) & 3);
    if (pairs) {
      const bool odd = lane & 1;
      auto neighbour = [](float x) {                      // the value lane l ^ 1 passes in
        return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
      };
      const int col0 = col_base - (odd ? 1 : 0);
#pragma unroll
      for (int i = 0; i < TA; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j) {
          const float got0 = neighbour(odd ? acc[i][j][0] : acc[i][j][2]);
          const float got1 = neighbour(odd ? acc[i][j][1] : acc[i][j][3]);
          const uint32_t w0 = odd ? Elem<Tag>::pack2(got0, acc[i][j][2]) : Elem<Tag>::pack2(acc[i][j][0], got0);
          const uint32_t w1 = odd ? Elem<Tag>::pack2(got1, acc[i][j][3]) : Elem<Tag>::pack2(acc[i][j][1], got1);
          const int row = row_base + i * 16 + (odd ? 2 : 0);
          const int col = col0 + j * 16;
          if (col < N) {
            if (row < M) *reinterpret_cast<uint32_t*>(C + (int64_t)row * ldc + col) = w0;
            if (row + 1 < M) *reinterpret_cast<uint32_t*>(C + (int64_t)(row + 1) * ldc + col) = w1;
          }
        }
      return;
    }
  }
  gemm_epilogue<Tag>([&](auto&& out) {
#pragma unroll
    for (int i = 0; i < TA; ++i)
#pragma unroll
      for (int j = 0; j < TB; ++j) {
        const int col = col_base + j * MS;
#pragma unroll
        for (int r = 0; r < (MS == 32 ? 16 : 4); ++r) {
          const int row = row_base + i * MS + (MS == 32 ? 8 * (r >> 2) + (r & 3) : r);
          if (row < M && col < N) out((int64_t)row * ldc + col, col, acc[i][j][r]);
        }
      }
  }, C, epi, bias);
}

bool gemm_pp_ok(const GemmArgs& g) {
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!al16(g.A) || !al16(g.B)) return false;
  if (g.K < 64 || g.K % 64 || g.lda % 8 || g.ldb % 8) return false;
  if (g.M < 1 || g.N < 1) return false;
  if (!g.transB && g.N % 8) return false;
  const int64_t lim = (int64_t)1 << 30;
  if (256 * g.lda >= lim) return false;
  if (g.transB ? 256 * g.ldb >= lim : 128 * g.ldb + g.N >= lim) return false;
  return true;
}

template <typename Tag, bool TRANSB, int MS, int BT, int BK>
static int launch_pp(const GemmArgs& g, hipStream_t s) {
  constexpr int PP_BM = BT, PP_BN = BT, PP_SMEM = PpTile<BT, BK>::SMEM;
  if (g.K % BK) return MLT_ERR_UNSUPPORTED;
  auto kern = gemm_pp_kernel<Tag, TRANSB, MS, BT, BK>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            PP_SMEM) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nbm = (int)((g.M + PP_BM - 1) / PP_BM), nbn = (int)((g.N + PP_BN - 1) / PP_BN);
  hipLaunchKernelGGL(kern, dim3(nbm * nbn), dim3(PP_NT), PP_SMEM, s, (int)g.M, (int)g.N, (int)g.K,
                     g.A, g.lda, g.B, g.ldb, g.C, g.ldc, nbm, nbn, device_xcds(), g.epi(), g.bias);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

// Only the 16x16x32 form is instantiated (MS = 16): measured on N(0,1) operands it runs 8-17 %
// faster than the 32x32x16 form of the same schedule (the chip is power-limited and this MFMA
// shape moves half as many accumulator registers per flop).
template <int BT, int BK>
static int run_pp_t(const GemmArgs& g, hipStream_t s) {
  constexpr int MS = 16;
  if (g.dtype == MLT_BF16)
    return g.transB ? launch_pp<bf16_tag, true, MS, BT, BK>(g, s) : launch_pp<bf16_tag, false, MS, BT, BK>(g, s);
  return g.transB ? launch_pp<f16_tag, true, MS, BT, BK>(g, s) : launch_pp<f16_tag, false, MS, BT, BK>(g, s);
}

int run_gemm_pp(const GemmArgs& g, int tile, int kstep, hipStream_t s) {
  if (tile == 128) return kstep == 128 ? run_pp_t<128, 128>(g, s) : run_pp_t<128, 64>(g, s);
  return run_pp_t<256, 64>(g, s);
}

}  // namespace mlt
