// GEMM C = A*B for gfx950, four wavefronts with 128 x 128 sub-tiles and a software-pipelined K loop.
//
// Same three levels as the paper's GEMM (arXiv 2503.14985, Sections 2.1-2.3: workgroup tile,
// per-warp sub-tile, hardware dot): workgroup tile 256 x 256, K step 64, 4 wavefronts as 2 x 2
// owning 128 x 128 each (the paper's "square" warp arrangement), MFMA 32x32x16. Against the
// 8-wavefront kernel of gemm_pp.hip (2 x 4 of 128 x 64) a wavefront reads 8 operand fragments from
// LDS per 16 MFMAs instead of 6 per 8: a third less LDS traffic per flop, which on this chip is
// power, and power is clock. The price is one wavefront per SIMD (its 256 accumulator registers
// leave no room for a second one), so nothing else hides latency: the loop is pipelined by hand.
// Measured: in shader clocks this kernel keeps the matrix pipes busy 73 % of the time (the 8-wave
// kernel 86 %) but clocks higher; the two come out within a few percent of each other, this one
// behind for B stored N x K, and it is not the default (MLT_GEMM_VARIANT=256w4 selects it). What
// it loses is the issue time of its own global loads: without them in the loop it runs 15 % faster,
// and the 8-wave kernel issues them from the wavefront that is not feeding the matrix pipe.
//   * a K step is 4 slices of 16 k; the 16 MFMAs of a slice are interleaved with the 8 (B stored
//     N x K) or 12 (B stored K x N, transposing reads) LDS reads of the NEXT slice's fragments
//     into a second fragment buffer, and with the global->LDS loads of later tiles;
//   * operand tiles go from global memory straight into LDS (global_load_lds_dwordx4) into a ring
//     of five 32 KB slots holding A_0 B_0 A_1 B_1 A_2 ... with the swizzles of gemm_pp.hip;
//   * one workgroup barrier per K step, placed between slices 2 and 3: by then every wavefront
//     has finished reading tile k (slice 3's fragments are in registers) and has seen its own
//     loads of tile k+1 land, so after the barrier slice 3 can prefetch slice 0 of tile k+1 and
//     the slots of tile k can be refilled; the loads are spread, one after every fourth MFMA:
//     B_{k+2} in slice 3 and the following slice 0, A_{k+3} in the slices 1 and 2 after that;
//   * the loop body has no branches: loads and prefetches past the last K step are issued all the
//     same, into slots nobody reads any more.
// Requirements as for gemm_pp.hip (K % 64 == 0, 16-byte aligned operands, 32-bit offsets).
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

constexpr int W4_BM = 256, W4_BN = 256, W4_BK = 64;
constexpr int W4_NT = 256;
constexpr int W4_SLOT = 32768;                           // one operand tile
constexpr int W4_NSLOT = 5;
constexpr int W4_SMEM = W4_NSLOT * W4_SLOT;              // 160 KB

}  // namespace

template <typename Tag, bool TRANSB>
__global__ __launch_bounds__(W4_NT) void gemm_w4_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc, int nbm,
    int nbn, int nxcd, int epi, const uint16_t* __restrict__ bias) {
  typedef typename Elem<Tag>::vec8 V8;
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;               // 2 x 2 wavefronts of 128 x 128
  int tile_m, tile_n;
  tile_of_block<8>(blockIdx.x, nbm, nbn, nxcd, tile_m, tile_n);
  const int m0 = tile_m * W4_BM, n0 = tile_n * W4_BN;

  // ---- global -> LDS assignments: a tile is 32 blocks of 1 KB; wavefront w fills blocks 8w ..
  // 8w+7 of every A tile and every B tile; lane l owns the 16-byte slot l of a block.
  const char* a_base = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
  const char* b_base;
  int64_t b_kstep;
  uint32_t voff_a[8], voff_b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = (wave * 8 + i) * 8 + (lane >> 3);          // tile row held by this slot
    const int c = (lane & 7) ^ ((r >> 1) & 7);               // k chunk stored in this slot
    const int rr = (m0 + r < M) ? r : (M - 1 - m0);
    voff_a[i] = (uint32_t)rr * (uint32_t)lda * 2u + (uint32_t)c * 16u;
  }
  if (TRANSB) {
    b_base = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
    b_kstep = W4_BK * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = (wave * 8 + i) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      const int rr = (n0 + r < N) ? r : (N - 1 - n0);
      voff_b[i] = (uint32_t)rr * (uint32_t)ldb * 2u + (uint32_t)c * 16u;
    }
  } else {
    b_base = reinterpret_cast<const char*>(B);
    b_kstep = (int64_t)W4_BK * ldb * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = (wave * 8 + i) * 2 + (lane >> 5);        // tile k row held by this slot
      const int q = (lane & 31) ^ (4 * (k & 3));             // n chunk stored in this slot
      const int col = n0 + q * 8;
      voff_b[i] = (uint32_t)k * (uint32_t)ldb * 2u + (uint32_t)(col < N ? col : 0) * 2u;
    }
  }
  const int KT = K / W4_BK;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  // Load i (0..7) of this wavefront's share of A_t (operand tile 2t) or B_t (operand tile 2t+1).
  // Tiles past the last K step are fetched all the same (from the last step's addresses, into
  // the slot they would have had, which nobody reads any more): the loop then needs no branch
  // between its MFMAs and every wait count is the same in every step.
  auto issue_a = [&](int t, int i) {
    const int ts = t < KT ? t : KT - 1;
    load_lds16(a_base + (int64_t)ts * (W4_BK * 2), voff_a[i],
                  lds0 + (uint32_t)((2 * t) % W4_NSLOT) * W4_SLOT + wave * 8192 + i * 1024);
  };
  auto issue_b = [&](int t, int i) {
    const int ts = t < KT ? t : KT - 1;
    load_lds16(b_base + (int64_t)ts * b_kstep, voff_b[i],
                  lds0 + (uint32_t)((2 * t + 1) % W4_NSLOT) * W4_SLOT + wave * 8192 + i * 1024);
  };

  // ---- fragment addresses (LDS byte addresses of slot 0; tile and k-slice steps are immediates)
  const int lq = lane & 31, h = lane >> 5;
  uint32_t a_adr[4], b_adr[4];
  {
    const int r = wm * 128 + lq;
    const int f = (lq >> 1) & 7;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) a_adr[kk] = lds0 + r * 128 + (((2 * kk + h) ^ f) * 16);
  }
  if (TRANSB) {
    const int r = wn * 128 + lq;
    const int f = (lq >> 1) & 7;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) b_adr[kk] = lds0 + r * 128 + (((2 * kk + h) ^ f) * 16);
  } else {
    // transposing read: 16-lane group g serves columns 16*(g%2).. of a 32-wide tile and k slots
    // 8*(g/2)..; lane s of the group addresses k row s/4 (+4 for the second read), columns 4*(s%4)..
    const int g = lane >> 4, s = lane & 15;
    const int krow = 8 * (g >> 1) + (s >> 2);
    const int x = 4 * (s >> 2);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int q = wn * 16 + 4 * j + 2 * (g & 1) + ((s & 3) >> 1);
      b_adr[j] = lds0 + krow * 512 + ((q ^ x) * 16) + 8 * (s & 1);
    }
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragments of k slice kk of the tiles in slots sa (A) and sb (B): A tile i / B tile j
  V8 fa[2][4], fb[2][4];
  auto read_a = [&](uint32_t sa, int kk, int i, V8& f) {
    f = __builtin_bit_cast(V8, *(const MLT_LDS u32x4*)(uintptr_t)(a_adr[kk] + sa + i * 32 * 128));
  };
  auto read_b = [&](uint32_t sb, int kk, int j, V8& f) {
    if (TRANSB) {
      f = __builtin_bit_cast(V8, *(const MLT_LDS u32x4*)(uintptr_t)(b_adr[kk] + sb + j * 32 * 128));
    } else {
      const uint32_t a = b_adr[j] + sb + kk * 16 * 512;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)a);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)(a + 4 * 512));
      f = join_tr<V8>(lo, hi);
    }
  };
#define W4_SB() __builtin_amdgcn_sched_barrier(0)

  // ---- prologue: operand tiles 0..3 (A_0 B_0 A_1 B_1), then wait for tile 0. (Step 0 fetches the
  // second half of B_1 once more, as every step does for its B_{k+1}: same data, same place.)
#pragma unroll
  for (int i = 0; i < 8; ++i) issue_a(0, i);
#pragma unroll
  for (int i = 0; i < 8; ++i) issue_b(0, i);
#pragma unroll
  for (int i = 0; i < 8; ++i) issue_a(1, i);
#pragma unroll
  for (int i = 0; i < 8; ++i) issue_b(1, i);
  __builtin_amdgcn_s_waitcnt(wait_imm(16, 15));
  MLT_BARRIER();
  W4_SB();
#pragma unroll
  for (int i = 0; i < 4; ++i) read_a(0, 0, i, fa[0][i]);
#pragma unroll
  for (int j = 0; j < 4; ++j) read_b(W4_SLOT, 0, j, fb[0][j]);
  W4_SB();

  uint32_t sa = 0, sb = W4_SLOT;                          // slot offsets of A_k and B_k
  for (int k = 0; k < KT; ++k) {
    const uint32_t sa_n = sa + 2 * W4_SLOT >= W4_SMEM ? sa + 2 * W4_SLOT - W4_SMEM : sa + 2 * W4_SLOT;
    const uint32_t sb_n = sb + 2 * W4_SLOT >= W4_SMEM ? sb + 2 * W4_SLOT - W4_SMEM : sb + 2 * W4_SLOT;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk == 3) {
        // tile k has been read completely (slice 3 sits in registers once lgkmcnt is 0); my loads
        // of tile k+1 must have landed; behind them only A_{k+2} may still be in flight
        __builtin_amdgcn_s_waitcnt(wait_imm(8, 0));
        MLT_BARRIER();
        W4_SB();
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = mfma32(fa[cur][i], fb[cur][j], acc[i][j]);
          W4_SB();
          const int n = i * 4 + j;                          // 0..15 within the slice
          // fragments of the next slice, one after every even MFMA
          // B tiles first (the next slice's first four MFMAs need all of them), then the A tiles
          const bool rd_b = n < 8, rd_a = n >= 8;
          const int rj = n >> 1, ri = (n - 8) >> 1;
          if (!(n & 1)) {
            if (kk < 3) {
              if (rd_a) read_a(sa, kk + 1, ri, fa[nxt][ri]);
              if (rd_b) read_b(sb, kk + 1, rj, fb[nxt][rj]);
            } else {                                        // (after the last step: fragments nobody uses)
              if (rd_a) read_a(sa_n, 0, ri, fa[nxt][ri]);
              if (rd_b) read_b(sb_n, 0, rj, fb[nxt][rj]);
            }
          }
          // global -> LDS loads of later tiles
          // one after every fourth MFMA: B_{k+1} in slice 3 of the previous step and slice 0, A_{k+2}
          // in slices 1 and 2
          if ((n & 3) == 3) {
            if (kk == 3) issue_b(k + 2, n >> 2);
            if (kk == 0) issue_b(k + 1, 4 + (n >> 2));
            if (kk == 1) issue_a(k + 2, n >> 2);
            if (kk == 2) issue_a(k + 2, 4 + (n >> 2));
          }
          W4_SB();
        }
    }
    sa = sa_n;
    sb = sb_n;
  }
#undef W4_SB
  __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));              // the surplus loads of the last steps

  // ---- epilogue: fp32 -> 16-bit (RNE) and store, or the other epilogue forms; guarded per element
  const int row_base = m0 + wm * 128 + 4 * h;
  const int col_base = n0 + wn * 128 + lq;
  gemm_epilogue<Tag>([&](auto&& out) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = col_base + j * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
          if (row < M && col < N) out((int64_t)row * ldc + col, col, acc[i][j][r]);
        }
      }
  }, C, epi, bias);
}

template <typename Tag, bool TRANSB>
static int launch_w4(const GemmArgs& g, hipStream_t s) {
  auto kern = gemm_w4_kernel<Tag, TRANSB>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            W4_SMEM) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nbm = (int)((g.M + W4_BM - 1) / W4_BM), nbn = (int)((g.N + W4_BN - 1) / W4_BN);
  hipLaunchKernelGGL(kern, dim3(nbm * nbn), dim3(W4_NT), W4_SMEM, s, (int)g.M, (int)g.N, (int)g.K,
                     g.A, g.lda, g.B, g.ldb, g.C, g.ldc, nbm, nbn, device_xcds(), g.epi(), g.bias);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

// same operand requirements as the two-group kernel (gemm_pp_ok)
int run_gemm_w4(const GemmArgs& g, hipStream_t s) {
  if (g.dtype == MLT_BF16)
    return g.transB ? launch_w4<bf16_tag, true>(g, s) : launch_w4<bf16_tag, false>(g, s);
  return g.transB ? launch_w4<f16_tag, true>(g, s) : launch_w4<f16_tag, false>(g, s);
}

}  // namespace mlt
