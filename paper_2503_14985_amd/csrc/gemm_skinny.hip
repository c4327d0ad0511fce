// Skinny GEMM C = A*B for gfx950: M <= 64 rows (next-token decode shapes, Section 4.1 of the paper
// (arXiv 2503.14985): memory-bound GEMMs with a small m), B given as the N x K row-major array
// (k contiguous). The whole cost is reading B once from HBM, so the kernel is built around that
// stream and nothing is staged in LDS:
//   * a workgroup owns 16, 32 or 64 columns of C (rows of the stored B; more when N is large, so
//     that an A fragment fetched from L2 serves more columns) and all of K; its 8 wavefronts
//     take the 32-wide K chunks round-robin, so at any moment the workgroup reads 512 contiguous
//     bytes of each of its 16 B rows;
//   * a lane loads 16 bytes (8 consecutive k) of one B row straight into the register that the
//     16x16x32 MFMA wants as its B operand (lane l: column l % 16, k slots 8*(l/16)..+7), and the
//     matching 16 bytes of one A row as the A operand; A (M x K, at most 64 rows) stays in L2;
//   * 16 KB of B per wavefront are in flight before the first MFMA of a batch;
//   * the 8 partial 16 x 16 fp32 tiles are added through LDS and rounded to 16 bit once.
// Requirements (host): transB, M <= 64, K % 8 == 0, lda % 8 == 0, ldb % 8 == 0, A and B 16-byte
// aligned. N and K need not be multiples of the tile.
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

constexpr int SK_NW = 8;            // wavefronts per workgroup = K split
constexpr int SK_NT = SK_NW * 64;
constexpr int SK_U = 16;            // chunks in flight per wavefront
constexpr int SK_MAXMT = 4;         // 16-row tiles of A (M <= 64)

template <typename Tag, int MT, int NT>
__global__ __launch_bounds__(SK_NT) void gemm_skinny_nt_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc) {
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int U = SK_U / NT;               // chunks per batch: 16 KB of B in flight per wavefront
  __shared__ float red[SK_NW][256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, q = lane >> 4;
  const int n0 = blockIdx.x * (16 * NT);
  const uint16_t* bp[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int nrow = n0 + nt * 16 + r16 < N ? n0 + nt * 16 + r16 : N - 1;   // clamped: never stored
    bp[nt] = B + (int64_t)nrow * ldb;
  }
  const uint16_t* ap[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int arow = mt * 16 + r16 < M ? mt * 16 + r16 : M - 1;
    ap[mt] = A + (int64_t)arow * lda;
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int KC = (K + 31) / 32;                            // 32-wide chunks; K % 8 == 0
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  for (int c0 = wave; c0 < KC; c0 += SK_NW * U) {
    // k of this lane's 8 values in chunk u of the batch; past K (last batch only) the loads
    // re-read k = 0 and the B values are zeroed after they have arrived
    const bool whole = (c0 + (U - 1) * SK_NW) * 32 + 32 <= K;   // wavefront-uniform
    u32x4 bfrag[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = (c0 + u * SK_NW) * 32 + 8 * q;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bfrag[u][nt] = *reinterpret_cast<const u32x4_mem*>(bp[nt] + ((whole || k < K) ? k : 0));
    }
    __builtin_amdgcn_sched_barrier(0);                     // all B loads of the batch go out first
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      u32x4 afrag[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = (c0 + u * SK_NW) * 32 + 8 * q;
        afrag[u] = *reinterpret_cast<const u32x4_mem*>(ap[mt] + ((whole || k < K) ? k : 0));
      }
      __builtin_amdgcn_sched_barrier(0);
      if (mt == 0 && !whole) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if ((c0 + u * SK_NW) * 32 + 8 * q >= K) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bfrag[u][nt] = zero4;
          }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = mfma16(__builtin_bit_cast(V8, afrag[u]), __builtin_bit_cast(V8, bfrag[u][nt]),
                               acc[mt][nt]);
    }
  }

  // one 16 x 16 tile at a time through LDS: lane owns C[4*q + r][r16] in acc[..][r]
  const int row = (tid & 255) >> 4, col = tid & 15;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) red[wave][(4 * q + r) * 16 + r16] = acc[mt][nt][r];
      __syncthreads();
      if (tid < 256) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < SK_NW; ++w) s += red[w][tid];
        const int gr = mt * 16 + row, gc = n0 + nt * 16 + col;
        if (gr < M && gc < N) C[(int64_t)gr * ldc + gc] = Elem<Tag>::from_f32(s);
      }
      __syncthreads();
    }
}

template <typename Tag, int MT, int NT>
int launch_skinny(const GemmArgs& g, hipStream_t s) {
  const unsigned nwg = (unsigned)((g.N + 16 * NT - 1) / (16 * NT));
  hipLaunchKernelGGL((gemm_skinny_nt_kernel<Tag, MT, NT>), dim3(nwg), dim3(SK_NT), 0, s, (int)g.M,
                     (int)g.N, (int)g.K, g.A, g.lda, g.B, g.ldb, g.C, g.ldc);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

// Columns per workgroup: more columns reuse each A fragment more often (A comes from L2 once per
// workgroup), fewer keep the chip full; at least ~2 workgroups per CU are wanted.
template <typename Tag, int MT>
int run_skinny_mt(const GemmArgs& g, hipStream_t s) {
  if (g.N >= 64 * 512) return launch_skinny<Tag, MT, 4>(g, s);
  if (g.N >= 32 * 512) return launch_skinny<Tag, MT, 2>(g, s);
  return launch_skinny<Tag, MT, 1>(g, s);
}

template <typename Tag>
int run_skinny_t(const GemmArgs& g, hipStream_t s) {
  switch ((g.M + 15) / 16) {
    case 1: return run_skinny_mt<Tag, 1>(g, s);
    case 2: return run_skinny_mt<Tag, 2>(g, s);
    case 3: return run_skinny_mt<Tag, 3>(g, s);
    case 4: return run_skinny_mt<Tag, 4>(g, s);
  }
  return MLT_ERR_UNSUPPORTED;
}

}  // namespace

// Worth it only when the columns alone fill the chip (one workgroup per 16 columns).
bool gemm_skinny_ok(const GemmArgs& g) {
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!g.transB || g.acc32 || g.M > 16 * SK_MAXMT || g.N < 1024) return false;
  if (!al16(g.A) || !al16(g.B)) return false;
  if (g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
  return true;
}

int run_gemm_skinny(const GemmArgs& g, hipStream_t s) {
  return g.dtype == MLT_BF16 ? run_skinny_t<bf16_tag>(g, s) : run_skinny_t<f16_tag>(g, s);
}

}  // namespace mlt
