// Attention forward O = softmax(scale * Q K^T [+ causal mask]) V for gfx950.
//
// Follows the FlashAttention-2 forward of the paper (arXiv 2503.14985, Section 2.5, Algorithm 1):
// Q is loaded once, K/V tiles stream through the loop, the two products sit back to back with an
// online softmax (running row maximum m and row sum l) in between, and the output tile is split
// over the wavefronts along its rows only, so no softmax statistic ever crosses a wavefront
// (the paper's "horizontal" partition: warpsPerCTA = [numWarps, 1]). The paper's layout table
// (Table 5) says P, the result of the first product, feeds the second product as an operand
// without being redistributed. On CDNA4 that holds if both products are computed transposed:
//
//   S^T = K_j Q^T      MFMA A operand = K_j rows (from LDS), B operand = Q^T (registers)
//   O^T += V_j^T P^T   MFMA A operand = V_j^T (LDS, transposing read), B operand = P^T
//
// A 32x32 MFMA accumulator gives lane l the column l%32 (one query) and 16 rows (keys); the B
// operand of the next MFMA wants, per lane, one column (the same query) and 8 values of the
// contraction index (keys). So the S^T accumulator registers, exponentiated and rounded to 16 bit,
// ARE the P^T operand: registers 0..7 feed one MFMA, 8..15 the next. The order in which keys
// fill the contraction slots is whatever the accumulator layout dictates; the V_j^T operand is
// fetched in that same order. Row statistics are per query, hence per lane: the row maximum needs
// one exchange with lane l^32 (the other half of the keys), the row sum none until the end, and
// the rescale of O^T by alpha is a plain per-lane multiply.
//
// Workgroup: 8 wavefronts x 32 query rows = 256 rows of one (batch, head); key tile 64.
#include <stdlib.h>
#include <string.h>

#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

constexpr int MHA_BM = 256;   // query rows per workgroup
constexpr int MHA_BN = 64;    // keys per loop step
constexpr int MHA_NW = 8;     // wavefronts per workgroup
constexpr int MHA_NT = MHA_NW * 64;

template <int D>
struct MhaLds {
  // K tile [BN][D + 8]: row stride 272 B (D = 128) / 144 B (D = 64): 16 consecutive rows at one
  // d offset fall in distinct 4-bank groups.
  // V tile [BN][D + 32]: row stride 320 B / 192 B, a multiple of 64 B that is 16 banks mod 64,
  // so the 4 key rows x 2 column halves of a transposing read cover all 64 banks once.
  static constexpr int KSTR = D + 8;
  static constexpr int VSTR = D + 32;
  static constexpr int K_BYTES = MHA_BN * KSTR * 2;
  static constexpr int V_BYTES = MHA_BN * VSTR * 2;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int SMEM = 2 * STAGE;
  static constexpr int CHUNKS = MHA_BN * (D / 8);        // 16-byte chunks per tile
  static constexpr int NLD = CHUNKS / MHA_NT;            // per thread, per matrix
  static_assert(CHUNKS % MHA_NT == 0, "tile must split evenly over threads");
};

// Combine a per-lane value with the one held by lane l ^ 32 (the lane that owns the other half
// of the keys of the same query). permlane32_swap exchanges the upper 32 lanes of its first
// operand with the lower 32 lanes of its second; fed the same register twice it returns the
// pair (lower-half values, upper-half values) in every lane, and max / + of the pair does not
// care which is which.
__device__ __forceinline__ float both_halves_max(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float both_halves_sum(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

// Workgroup id -> (batch*head, query tile). Consecutive ids go round-robin to the 8 XCDs; undo
// that so each XCD owns a contiguous range of logical ids, then let consecutive logical ids walk
// the query tiles of one head, last tile first (with the causal mask the last tile has the most
// work). All tiles of a head then run on one XCD close in time and share its K/V in that L2.
__device__ __forceinline__ void mha_block_map(int bid, int total, int nq, int& bh, int& qt) {
  constexpr int NXCD = 8;
  const int q = total / NXCD, rem = total % NXCD;
  const int xcd = bid % NXCD, idx = bid / NXCD;
  const int logical = xcd * q + (xcd < rem ? xcd : rem) + idx;
  bh = logical / nq;
  qt = nq - 1 - logical % nq;
}

template <typename Tag, int D, bool CAUSAL>
__global__ __launch_bounds__(MHA_NT) void mha_fwd_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, uint16_t* __restrict__ O, int Sq, int Sk, int nq, int total,
    float c, int negate) {
  typedef MhaLds<D> L;
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int NKK = D / 16;     // k slices of the first product (contraction over d)
  constexpr int NDT = D / 32;     // 32-row tiles of O^T
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, h = lane >> 5;
  int bh, qt;
  mha_block_map(blockIdx.x, total, nq, bh, qt);
  const int q0 = qt * MHA_BM + wave * 32;               // first query row of this wavefront
  const int my_q = q0 + lq;

  const uint16_t* Qh = Q + (int64_t)bh * Sq * D;
  const uint16_t* Kh = K + (int64_t)bh * Sk * D;
  const uint16_t* Vh = V + (int64_t)bh * Sk * D;

  // Keys this workgroup has to look at. Causal, top-left aligned: key j is visible to query i
  // iff j <= i, so nothing beyond the last query row of the tile is needed.
  int kv_len = Sk;
  if (CAUSAL) {
    const int last_q = (qt + 1) * MHA_BM < Sq ? (qt + 1) * MHA_BM : Sq;   // exclusive
    kv_len = last_q < Sk ? last_q : Sk;
  }
  const int nblk = (kv_len + MHA_BN - 1) / MHA_BN;

  // ---- Q^T operand, resident in registers: query lq, d = 16*kk + 8*h .. +7
  V8 qf[NKK];
  {
    const int row = my_q < Sq ? my_q : Sq - 1;
    const uint16_t* qp = Qh + (int64_t)row * D + 8 * h;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const u32x4 raw = *reinterpret_cast<const u32x4_mem*>(qp + kk * 16);
      qf[kk] = __builtin_bit_cast(V8, raw);
    }
  }

  // ---- K/V staging: thread handles chunks tid + i*NT of the [BN][D/8] chunk grid
  constexpr int DC = D / 8;
  const int ld_row = tid / DC, ld_dc = (tid % DC) * 8;
  constexpr int ROW_STEP = MHA_NT / DC;
  u32x4 gk[L::NLD], gv[L::NLD];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  auto load_kv = [&](int blk) {
#pragma unroll
    for (int i = 0; i < L::NLD; ++i) {
      const int key = blk * MHA_BN + ld_row + i * ROW_STEP;
      const bool ok = key < Sk;
      const int64_t off = (int64_t)(ok ? key : Sk - 1) * D + ld_dc;
      gk[i] = *reinterpret_cast<const u32x4_mem*>(Kh + off);
      const u32x4 v = *reinterpret_cast<const u32x4_mem*>(Vh + off);
      gv[i] = ok ? v : zero4;      // rows past Sk get weight 0; keep 0 * V finite
    }
  };
  auto store_kv = [&](int stage) {
    char* base = smem + stage * L::STAGE;
#pragma unroll
    for (int i = 0; i < L::NLD; ++i) {
      const int row = ld_row + i * ROW_STEP;
      *reinterpret_cast<u32x4_mem*>(base + (row * L::KSTR + ld_dc) * 2) = gk[i];
      *reinterpret_cast<u32x4_mem*>(base + L::K_BYTES + (row * L::VSTR + ld_dc) * 2) = gv[i];
    }
  };

  // ---- fragment addresses
  // K rows as MFMA A operand: key row lq of a 32-key sub-tile, d = 16*kk + 8*h
  const int k_frag = (lq * L::KSTR + 8 * h) * 2;
  // V^T as MFMA A operand through the transposing read: 16-lane group g = lane/16 serves output
  // rows d = 16*(g%2) + i and contraction half h = g/2; lane s of the group addresses key row
  // 4*h + s/4 and d columns 4*(s%4)..+3.
  const int vg = lane >> 4, vs = lane & 15;
  const int v_frag = L::K_BYTES + ((4 * (vg >> 1) + (vs >> 2)) * L::VSTR + 16 * (vg & 1) + 4 * (vs & 3)) * 2;

  f32x16 o_acc[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
  float m_run = -__builtin_inff();   // running maximum of the raw (unscaled, sign-adjusted) scores
  float l_run = 0.f;                 // running sum over this lane's half of the keys

  // K fragments are fetched in chunks of KCH slices, one chunk ahead of the MFMAs that use them;
  // V^T fragments per group of 16 keys (NDT MFMAs), one group ahead.
  constexpr int KCH = 4;
  constexpr int CPK = NKK / KCH;          // chunks per 32-key sub-tile
  constexpr int NKC = 2 * CPK;            // chunks per key tile
  static_assert(NKK % KCH == 0 && NKC % 2 == 0, "chunking of the first product");
  auto load_kchunk = [&](const char* st, int ch, V8 (&kf)[KCH]) {
    const int kb = ch / CPK, kk0 = (ch % CPK) * KCH;
#pragma unroll
    for (int i = 0; i < KCH; ++i)
      kf[i] = lds_read8<V8>(st, k_frag + (kb * 32 * L::KSTR + (kk0 + i) * 16) * 2);
  };
  auto load_vgroup = [&](const char* st, int g, V8 (&vf)[NDT]) {
    const int vrow = g * 16 * L::VSTR * 2;                 // keys 16*g .. 16*g + 15 of the tile
#pragma unroll
    for (int t = 0; t < NDT; ++t) {
      const int off = v_frag + vrow + t * 32 * 2;
      const s16x4 lo = lds_read_tr4(st, off);
      const s16x4 hi = lds_read_tr4(st, off + 8 * L::VSTR * 2);
      vf[t] = join_tr<V8>(lo, hi);
    }
  };

  load_kv(0);
  store_kv(0);
  if (nblk > 1) load_kv(1);
  __syncthreads();

  V8 kf[2][KCH], vf[2][NDT];
  load_kchunk(smem, 0, kf[0]);

  for (int j = 0; j < nblk; ++j) {
    const int cur = j & 1;
    const char* st = smem + cur * L::STAGE;
    const int kb0 = j * MHA_BN;
    // Causal: a wavefront whose last row is above this key block has nothing visible in it.
    const bool active = !CAUSAL || (kb0 <= q0 + 31);

    f32x16 s_acc[2];
    if (active) {
      // ---- S^T = K_j Q^T  (two 32-key sub-tiles)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[kb][r] = 0.f;
#pragma unroll
      for (int ch = 0; ch < NKC; ++ch) {
        if (ch + 1 < NKC) load_kchunk(st, ch + 1, kf[(ch + 1) & 1]);
        else load_vgroup(st, 0, vf[0]);                    // first V group rides along
        __builtin_amdgcn_sched_barrier(0);
        const int kb = ch / CPK, kk0 = (ch % CPK) * KCH;
#pragma unroll
        for (int i = 0; i < KCH; ++i) s_acc[kb] = mfma32(kf[ch & 1][i], qf[kk0 + i], s_acc[kb]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // Tile j+1 (in registers since the previous step) goes to the other stage; the registers
    // are refilled with tile j+2. Safe: everyone left that stage at the previous barrier.
    if (j + 1 < nblk) {
      store_kv(cur ^ 1);
      if (j + 2 < nblk) load_kv(j + 2);
    }

    if (active) {
      // ---- online softmax on the 32 scores this lane holds for its query
      if (negate) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) s_acc[kb][r] = -s_acc[kb][r];
      }
      // register r of sub-tile kb is key kb0 + 32*kb + 8*(r/4) + 4*h + r%4
      const bool need_mask = (CAUSAL && (kb0 + MHA_BN - 1 > q0)) || (kb0 + MHA_BN > Sk);
      const int limit = CAUSAL ? (my_q < Sk - 1 ? my_q : Sk - 1) : Sk - 1;     // last visible key
      const int key_base = kb0 + 4 * h;
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (key_base + 32 * kb + 8 * (r >> 2) + (r & 3) > limit) s_acc[kb][r] = -__builtin_inff();
      }
      float mx = s_acc[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = __builtin_fmaxf(mx, s_acc[kb][r]);
      mx = both_halves_max(mx);
      const float m_new = __builtin_fmaxf(m_run, mx);
      // Rescale only when some row of this wavefront has a new maximum (alpha is 1 otherwise).
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = (m_run == -__builtin_inff()) ? 0.f : __builtin_amdgcn_exp2f((m_run - m_new) * c);
        l_run *= alpha;
#pragma unroll
        for (int t = 0; t < NDT; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) o_acc[t][r] *= alpha;
        m_run = m_new;
      }
      const float mc = m_run * c;
      float psum = 0.f;
      if (need_mask) {
        // the exponent of a masked score may be NaN (c = 0): select the weight, never compute it
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r], c, -mc));
            if (key_base + 32 * kb + 8 * (r >> 2) + (r & 3) > limit) p = 0.f;
            s_acc[kb][r] = p;
            psum += p;
          }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r], c, -mc));
            s_acc[kb][r] = p;
            psum += p;
          }
      }
      l_run += psum;

      // ---- O^T += V_j^T P^T : per 16 keys (group g) one MFMA per 32-row tile of O^T
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (g + 1 < 4) load_vgroup(st, g + 1, vf[(g + 1) & 1]);
        u32x4 pw;
#pragma unroll
        for (int w = 0; w < 4; ++w)
          pw[w] = Elem<Tag>::pack2(s_acc[g >> 1][8 * (g & 1) + 2 * w], s_acc[g >> 1][8 * (g & 1) + 2 * w + 1]);
        const V8 pf = __builtin_bit_cast(V8, pw);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NDT; ++t) o_acc[t] = mfma32(vf[g & 1][t], pf, o_acc[t]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
    if (j + 1 < nblk) load_kchunk(smem + (cur ^ 1) * L::STAGE, 0, kf[0]);
  }

  // ---- epilogue: O = O^T / l, l summed over both key halves; 4 consecutive d per store
  const float l_tot = both_halves_sum(l_run);
  const float inv = 1.f / l_tot;
  if (my_q < Sq) {
    uint16_t* op = O + ((int64_t)bh * Sq + my_q) * D + 4 * h;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = Elem<Tag>::pack2(o_acc[t][4 * g] * inv, o_acc[t][4 * g + 1] * inv);
        w[1] = Elem<Tag>::pack2(o_acc[t][4 * g + 2] * inv, o_acc[t][4 * g + 3] * inv);
        *reinterpret_cast<u32x2_mem*>(op + t * 32 + 8 * g) = w;
      }
  }
}

template <typename Tag, int D, bool CAUSAL>
int launch_mha(const MhaArgs& a, hipStream_t s) {
  typedef MhaLds<D> L;
  auto kern = mha_fwd_kernel<Tag, D, CAUSAL>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            L::SMEM) != hipSuccess) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nq = (int)((a.Sq + MHA_BM - 1) / MHA_BM);
  const int64_t total = a.B * a.H * nq;
  if (total > 0x7fffffff) return MLT_ERR_UNSUPPORTED;
  const float LOG2E = 1.4426950408889634f;
  const float c = (a.scale < 0 ? -a.scale : a.scale) * LOG2E;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(MHA_NT), L::SMEM, s, a.Q, a.K, a.V, a.O,
                     (int)a.Sq, (int)a.Sk, nq, (int)total, c, a.scale < 0 ? 1 : 0);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

template <typename Tag>
int run_mha_t(const MhaArgs& a, hipStream_t s) {
  if (a.D == 128) return a.causal ? launch_mha<Tag, 128, true>(a, s) : launch_mha<Tag, 128, false>(a, s);
  if (a.D == 64) return a.causal ? launch_mha<Tag, 64, true>(a, s) : launch_mha<Tag, 64, false>(a, s);
  return MLT_ERR_UNSUPPORTED;
}

}  // namespace

MhaPlan plan_mha(const MhaArgs& a) {
  MhaPlan p;
  if (a.D != 64 && a.D != 128) return p;
  p.supported = true;
  p.bm = MHA_BM; p.bn = MHA_BN; p.waves = MHA_NW;
  // Tuning/debug override: MLT_MHA_VARIANT = single selects the older single-schedule kernel,
  // pp32 / pp16 the two-group kernel on 32x32x16 / 16x16x32 MFMAs, ps its persistent form (unmasked
  // problems with at least two key tiles per item; other problems fall back to pp32).
  const char* e = getenv("MLT_MHA_VARIANT");
  p.two_group = mha_pp_ok(a) && !(e && !strcmp(e, "single"));
  if (p.two_group) {
    // Default: 32x32x16. Measured for D = 128: the 16x16x32 form is 3 % faster in back-to-back
    // launches but 2 % slower when it alternates with the GEMM (the benchmark step); for D = 64 it
    // does not fit the 128 registers that let two workgroups share a CU (-6 %).
    p.mfma_size = 32;
    if (e && !strcmp(e, "pp16")) p.mfma_size = 16;
    if (e && !strcmp(e, "pp32")) p.mfma_size = 32;
    // The persistent form ("ps" forces it wherever it applies). Measured, unmasked, 2048 items,
    // time per item against the per-item kernel: D = 128 gains 25 % at 2 key tiles per item, 8 %
    // at 4, 3 % at 8 and loses 1.5 % at 16, 3 % at 32 and 4 % at 64 (its loop carries the item
    // bookkeeping). D = 64 has no persistent form (mha_ps_ok).
    const bool ps_pays = a.Sk <= 8 * 64;
    p.persistent = mha_ps_ok(a) && (e ? !strcmp(e, "ps") : ps_pays);
    if (p.persistent) {
      p.name = "mha_fwd_d128_256x64_ps";
      return p;
    }
    if (p.mfma_size == 16) {
      if (a.D == 128) p.name = a.causal ? "mha_fwd_d128_causal_256x64_pp16" : "mha_fwd_d128_256x64_pp16";
      else p.name = a.causal ? "mha_fwd_d64_causal_256x64_pp16" : "mha_fwd_d64_256x64_pp16";
    } else {
      if (a.D == 128) p.name = a.causal ? "mha_fwd_d128_causal_256x64_pp" : "mha_fwd_d128_256x64_pp";
      else p.name = a.causal ? "mha_fwd_d64_causal_256x64_pp" : "mha_fwd_d64_256x64_pp";
    }
    return p;
  }
  if (a.D == 128) p.name = a.causal ? "mha_fwd_d128_causal_256x64" : "mha_fwd_d128_256x64";
  else p.name = a.causal ? "mha_fwd_d64_causal_256x64" : "mha_fwd_d64_256x64";
  return p;
}

int run_mha(const MhaArgs& a, const MhaPlan& p, hipStream_t s) {
  if (p.persistent) return run_mha_ps(a, s);
  if (p.two_group) return run_mha_pp(a, p.mfma_size, s);
  return a.dtype == MLT_BF16 ? run_mha_t<bf16_tag>(a, s) : run_mha_t<f16_tag>(a, s);
}

}  // namespace mlt
