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
        bfrag[u][nt] = load_stream16(bp[nt] + ((whole || k < K) ? k : 0));   // B is read once
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


// ---------------------------------------------------------------------------------------------
// Streaming variant for large B. What limits the kernel above on matrices far beyond the caches
// is the shape of its HBM requests (one load instruction touches 16 rows with 64 bytes each) and,
// for taller A, that A is fetched from L2 again for every 16 columns. Here B goes through an LDS
// ring in long contiguous row pieces and stays 7 stages (112 KB per CU) in flight:
//   * a stage is 16 KB of B: 16 rows x 512 k (1 KB per row, one row per load instruction: 64 lanes
//     x 16 contiguous bytes, global_load_lds_dwordx4). (A wider stage of 64 rows x 128 k, which
//     reuses every A fragment for four column tiles, measured slower than the small-tile kernels
//     wherever it beat this one, and is no longer built.) The ring holds 8 stages (128 KB);
//   * wavefronts 0-3 only fetch: wavefront p issues load instructions 4p .. 4p+3 of every stage,
//     seven stages ahead. Their vector-memory counter sees nothing but these loads, so "stage s
//     has landed" is an exact count; wavefronts 4-7 only compute: they split the 32-wide k chunks
//     of a stage among themselves, read the B fragments from LDS and the A fragments from global
//     memory (A stays in L2; their loads are counted by the compiler as usual);
//   * one workgroup barrier per stage; the slot of stage s-1 is refilled right after barrier s;
//   * workgroups are persistent (one per CU) and walk over their column blocks without letting
//     the ring drain; at the end of a block the four partial tiles are added through a separate
//     LDS area and stored;
//   * within a row piece the 16-byte chunks are stored permuted (chunk c at position c ^ (row &
//     15)): the source address of a lane is free, its LDS position is not, and the 16 lanes that
//     read 16 rows at one k position must hit 16 distinct bank groups.
constexpr int SD_ST = 8;              // ring stages
constexpr int SD_STAGE_B = 16384;     // bytes of B per stage
constexpr int SD_SMEM = SD_ST * SD_STAGE_B;
constexpr int SD_RED = 4 * 4 * 256 * 4;   // reduction area behind the ring: [4 wavefronts][4 tiles][256]

struct SdCfg {
  static constexpr int RPS = 16;                 // rows of B (columns of C) per stage and column block
  static constexpr int KS = 512;                 // k values per stage
  static constexpr int PB = KS * 2;              // bytes of a row piece
  static constexpr int LPR = PB / 16;            // lanes per row piece
  static constexpr int NT = RPS / 16;            // 16-column tiles per block
  static constexpr int J = KS / 32 / 4;          // k chunks per computing wavefront and stage
};

template <typename Tag, int MT>
__global__ __launch_bounds__(SK_NT) void gemm_skinny_dma_kernel(
    int M, int N, int K, const uint16_t* __restrict__ A, int64_t lda,
    const uint16_t* __restrict__ B, int64_t ldb, uint16_t* __restrict__ C, int64_t ldc) {
  typedef typename Elem<Tag>::vec8 V8;
  typedef SdCfg L;
  constexpr int KS = L::KS, NT = L::NT, J = L::J;
  extern __shared__ __align__(16) char smem[];             // the ring, then the reduction area
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int NS = (K + KS - 1) / KS;                        // stages per column block
  const int nblocks = (N + L::RPS - 1) / L::RPS;
  // Persistent workgroups: this one owns column blocks blockIdx.x, + gridDim.x, ... and takes
  // them in groups of up to GB. The stages of a group are ordered k stage first: (k stage 0 of
  // every block of the group), (k stage 1 of every block), ...; the accumulators of all the
  // group's blocks stay in registers, and the A fragments of a k stage are fetched once per group
  // instead of once per block. All stages of all groups form one stream g = 0 .. G-1, so the ring
  // never drains between blocks or groups.
  // (as many as the registers take: 8 blocks for one 16-row tile of A in the narrow form)
  constexpr int GB = MT == 1 ? 8 : MT == 2 ? 4 : 2;
  const int nmine = (nblocks - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  const int G = nmine * NS;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

  if (wave < 4) {
    // ---- fetching wavefronts: load instruction ii of a stage fills LDS bytes ii*1024 .. +1023 of
    // the slot, i.e. rows ii*(64/LPR) .. of the stage; lane l serves row l / LPR of those at
    // position l % LPR. The cursor (i_*) names the next stage of the stream to fetch.
    int i_g = 0, i_base = 0, i_nb = nmine < GB ? nmine : GB, i_ks = 0, i_b = 0;
    auto issue_next = [&]() __attribute__((always_inline)) {
      if (i_g >= G) return;
      const int n0 = ((int)blockIdx.x + (i_base + i_b) * (int)gridDim.x) * L::RPS;
      const int k0 = i_ks * KS;
      const char* Bw = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
      const uint32_t slot = lds0 + (uint32_t)(i_g % SD_ST) * SD_STAGE_B;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ii = wave * 4 + i;
        const int r = ii * (64 / L::LPR) + lane / L::LPR;
        const int nrow = n0 + r < N ? r : N - 1 - n0;      // clamped: such columns are never stored
        int ck = (lane % L::LPR) ^ (r & 15);               // the 16-byte chunk this lane fetches
        if (k0 + ck * 8 >= K) ck = 0;                      // past K (last stage): any valid chunk, zeroed later
        load_lds16_stream(Bw, (uint32_t)nrow * (uint32_t)ldb * 2u + (uint32_t)(k0 + ck * 8) * 2u,
                      slot + (uint32_t)ii * 1024u);
      }
      ++i_g;
      if (++i_b == i_nb) {
        i_b = 0;
        if (++i_ks == NS) {
          i_ks = 0;
          i_base += GB;
          i_nb = nmine - i_base < GB ? nmine - i_base : GB;
        }
      }
    };
#pragma unroll
    for (int t = 0; t < SD_ST - 1; ++t) issue_next();
    int g = 0;
    for (int base = 0; base < nmine; base += GB) {
      const int nb = nmine - base < GB ? nmine - base : GB;
      for (int t = 0; t < NS * nb; ++t, ++g) {
        // issued so far: stages 0 .. min(G, g + SD_ST - 1) - 1; those after g may stay in flight
        const int last = g + SD_ST - 2 < G - 1 ? g + SD_ST - 2 : G - 1;
        switch (last - g) {
          case 0: __builtin_amdgcn_s_waitcnt(wait_imm(0, 15)); break;
          case 1: __builtin_amdgcn_s_waitcnt(wait_imm(4, 15)); break;
          case 2: __builtin_amdgcn_s_waitcnt(wait_imm(8, 15)); break;
          case 3: __builtin_amdgcn_s_waitcnt(wait_imm(12, 15)); break;
          case 4: __builtin_amdgcn_s_waitcnt(wait_imm(16, 15)); break;
          case 5: __builtin_amdgcn_s_waitcnt(wait_imm(20, 15)); break;
          default: __builtin_amdgcn_s_waitcnt(wait_imm(24, 15)); break;
        }
        MLT_BARRIER();                      // stage g is complete in LDS for everyone
        issue_next();                                      // stage g + SD_ST - 1, into the slot of stage g-1 (read before this barrier)
      }
      // end of a group: the barriers of the computing wavefronts' reductions (two per block and
      // row tile, less the very first)
      for (int t = 0; t < 2 * nb * MT - 1; ++t) __syncthreads();
    }
  } else {
    // ---- computing wavefronts: wavefront cw takes k chunks J*cw .. J*cw + J-1 of every stage
    const int cw = wave - 4, ctid = tid - 256;
    const int r16 = lane & 15, q = lane >> 4;
    float* red = reinterpret_cast<float*>(smem + SD_SMEM);  // [4][NT][256]
    const uint16_t* ap[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int arow = mt * 16 + r16 < M ? mt * 16 + r16 : M - 1;
      ap[mt] = A + (int64_t)arow * lda;
    }
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    f32x4 acc[GB][MT][NT];
#pragma unroll
    for (int gb = 0; gb < GB; ++gb)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[gb][mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // A fragments of k stage ks: k = ks*KS + (J*cw + j)*32 + 8*q
    auto load_a = [&](int ks, u32x4 (&af)[J][MT]) __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int k = ks * KS + (J * cw + j) * 32 + 8 * q;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          af[j][mt] = *reinterpret_cast<const u32x4_mem*>(ap[mt] + (k < K ? k : 0));
      }
    };
    int g = 0;
    u32x4 af0[J][MT], af1[J][MT];
    load_a(0, af0);
    for (int base = 0; base < nmine; base += GB) {
      const int nb = nmine - base < GB ? nmine - base : GB;
      // k stage ks of every block of the group: `cur` holds its A fragments; those of the next k
      // stage (of this group, or stage 0 for the next group) are requested into `nxt` meanwhile
      auto k_stage = [&](int ks, u32x4 (&cur)[J][MT], u32x4 (&nxt)[J][MT]) __attribute__((always_inline)) {
        const bool whole = (ks + 1) * KS <= K;
#pragma unroll
        for (int gb = 0; gb < GB; ++gb) {
          if (gb < nb) {
            MLT_BARRIER();
            const uint32_t slot = lds0 + (uint32_t)(g % SD_ST) * SD_STAGE_B;
            u32x4 bf[J][NT];
#pragma unroll
            for (int j = 0; j < J; ++j) {
              const int c16 = (J * cw + j) * 4 + q;              // 16-byte chunk of the row piece
#pragma unroll
              for (int nt = 0; nt < NT; ++nt)
                bf[j][nt] = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(
                    slot + (uint32_t)(nt * 16 + r16) * L::PB + (uint32_t)((c16 ^ r16) << 4));
            }
            if (gb == 0) load_a(ks + 1 < NS ? ks + 1 : 0, nxt);  // unconditional: keeps the load counting exact
#pragma unroll
            for (int j = 0; j < J; ++j) {
              const bool dead = !whole && ks * KS + (J * cw + j) * 32 + 8 * q >= K;
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                const u32x4 a = dead ? zero4 : cur[j][mt];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                  const u32x4 bb = dead ? zero4 : bf[j][nt];
                  acc[gb][mt][nt] = mfma16(__builtin_bit_cast(V8, a), __builtin_bit_cast(V8, bb), acc[gb][mt][nt]);
                }
              }
            }
            ++g;
          }
        }
      };
      for (int ks = 0; ks < NS; ks += 2) {
        k_stage(ks, af0, af1);
        if (ks + 1 < NS) k_stage(ks + 1, af1, af0);
      }
      if (NS & 1) {
        // an odd number of k stages leaves the fragments of the next group's stage 0 in af1
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) af0[j][mt] = af1[j][mt];
      }
      // end of a group: per block and 16-row tile of A the four wavefronts' partial tiles meet in
      // LDS, 256 lanes add them and store (2 * nb * MT - 1 barriers, matched by the fetching
      // wavefronts)
#pragma unroll
      for (int gb = 0; gb < GB; ++gb) {
        if (gb < nb) {
          const int n0 = ((int)blockIdx.x + (base + gb) * (int)gridDim.x) * L::RPS;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            if (gb > 0 || mt > 0) __syncthreads();             // the previous sums have been read
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                red[(cw * NT + nt) * 256 + (4 * q + r) * 16 + r16] = acc[gb][mt][nt][r];
                acc[gb][mt][nt][r] = 0.f;
              }
            __syncthreads();                                   // with the fence: the partial tiles are LDS stores
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              float sum = 0.f;
#pragma unroll
              for (int w = 0; w < 4; ++w) sum += red[(w * NT + nt) * 256 + ctid];
              const int gr = mt * 16 + (ctid >> 4), gc = n0 + nt * 16 + (ctid & 15);
              if (gr < M && gc < N) C[(int64_t)gr * ldc + gc] = Elem<Tag>::from_f32(sum);
            }
          }
        }
      }
    }
  }
}

template <typename Tag, int MT>
int launch_skinny_dma(const GemmArgs& g, hipStream_t s) {
  auto kern = gemm_skinny_dma_kernel<Tag, MT>;
  static thread_local int configured_dev = -1;            // opt in to > 64 KB LDS once per device
  static thread_local int ncu = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            SD_SMEM + SD_RED) != hipSuccess ||
        hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int64_t nblocks = (g.N + SdCfg::RPS - 1) / SdCfg::RPS;
  const unsigned nwg = (unsigned)(nblocks < ncu ? nblocks : ncu);   // one persistent workgroup per CU
  hipLaunchKernelGGL(kern, dim3(nwg), dim3(SK_NT), SD_SMEM + SD_RED, s, (int)g.M, (int)g.N, (int)g.K,
                     g.A, g.lda, g.B, g.ldb, g.C, g.ldc);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

template <typename Tag>
int run_skinny_dma_t(const GemmArgs& g, hipStream_t s) {
  switch ((g.M + 15) / 16) {
    case 1: return launch_skinny_dma<Tag, 1>(g, s);
    case 2: return launch_skinny_dma<Tag, 2>(g, s);
    case 3: return launch_skinny_dma<Tag, 3>(g, s);
    case 4: return launch_skinny_dma<Tag, 4>(g, s);
  }
  return MLT_ERR_UNSUPPORTED;
}

}  // namespace

// Worth it only when the columns alone fill the chip (one workgroup per 16 columns).
bool gemm_skinny_ok(const GemmArgs& g) {
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  if (!g.transB || g.acc32 || g.fused() || g.M > 16 * SK_MAXMT || g.N < 1024) return false;
  if (!al16(g.A) || !al16(g.B)) return false;
  if (g.K % 8 || g.lda % 8 || g.ldb % 8) return false;
  return true;
}

int run_gemm_skinny(const GemmArgs& g, hipStream_t s) {
  return g.dtype == MLT_BF16 ? run_skinny_t<bf16_tag>(g, s) : run_skinny_t<f16_tag>(g, s);
}

// The streaming variant addresses B rows with 32-bit byte offsets from the column block's first row.
bool gemm_skinny_dma_ok(const GemmArgs& g) {
  return gemm_skinny_ok(g) && g.ldb * 2 * 64 + g.K * 2 < ((int64_t)1 << 32);
}

int run_gemm_skinny_dma(const GemmArgs& g, hipStream_t s) {
  return g.dtype == MLT_BF16 ? run_skinny_dma_t<bf16_tag>(g, s) : run_skinny_dma_t<f16_tag>(g, s);
}

}  // namespace mlt
