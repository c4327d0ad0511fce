// Paged attention for decoding (arXiv 2503.14985, Section 3.2) for gfx950: one query per
// (sequence, head) over that sequence's keys and values, which live in fixed-size blocks of a cache
// and are found through a per-sequence block table.
//
// The paper's point about this kernel is its warp distribution: with a single query row there is
// nothing to split along the rows, so the KEYS are split over the warps of a workgroup, every warp
// runs the FlashAttention recurrence on its own cache blocks, and the partial maxima, sums and
// outputs are reduced across warps through shared local memory to one warp that stores the
// result (Listing 6). The same decomposition here, one level finer: a workgroup of 4 wavefronts
// owns one (sequence, head); the keys are cut into units of 16, wavefront w takes units w, w+4,
// ...; inside a wavefront each group of D/8 lanes owns one key row of a load (4 rows per 1 KB
// load for D = 128, 8 for D = 64) and keeps its OWN running maximum, sum and output slice, so
// nothing is exchanged between lanes except the D/8-lane sum of a dot product. All partial
// results (16 or 32 per workgroup) meet once, in LDS, at the end.
//
// With fewer (sequence, head) pairs than the chip needs workgroups, the same split goes one level
// up as well: the units of a sequence are cut into `nsplit` contiguous ranges, one workgroup per
// (sequence, head, range); each leaves its maximum, sum and unnormalised output slice (fp32) in a
// scratch buffer, and a second small kernel merges the ranges of a pair in index order, the way
// the workgroup merges its own partial results.
//
// The operation is bound by reading the cache once from HBM (2 * seq_len * D * 2 bytes per
// sequence and head), so there is no MFMA here (a 1-row product would waste it) and no LDS staging:
// 16-byte loads go straight to registers, one unit ahead of the arithmetic. Products use the
// packed dot instructions (v_dot2_f32_bf16 / v_dot2_f32_f16): q.k as four of them per lane and key,
// p.v as one per output element with the weight, rounded to the 16-bit type as in Listing 5's
// p.to(float16), in one half of the second operand.
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

constexpr int PG_NW = 4;            // wavefronts per workgroup
constexpr int PG_NT = PG_NW * 64;
constexpr int PG_UNIT = 16;         // keys per unit

// sum over the 16 (or 8) lanes that share a key row; every lane of the group gets the total
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, false));  // row_half_mirror
  if (LPR == 16)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, false));  // row_mirror
  return x;
}

template <typename Tag> struct Dot2;
template <> struct Dot2<bf16_tag> {
  static __device__ __forceinline__ float f(uint32_t a, uint32_t b, float c) {
    typedef __attribute__((ext_vector_type(2))) __bf16 v2;
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2, a), __builtin_bit_cast(v2, b), c, false);
  }
};
template <> struct Dot2<f16_tag> {
  static __device__ __forceinline__ float f(uint32_t a, uint32_t b, float c) {
    typedef __attribute__((ext_vector_type(2))) _Float16 v2;
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(v2, a), __builtin_bit_cast(v2, b), c, false);
  }
};

// SPLIT: blockIdx.y is the range of units this workgroup takes, and the result goes to `part`
// ([pair][range][2 + D] floats: maximum (log2 domain), sum, unnormalised outputs) instead of O.
template <typename Tag, int D, bool SPLIT>
__global__ __launch_bounds__(PG_NT) void paged_decode_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kc,
    const uint16_t* __restrict__ Vc, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, uint16_t* __restrict__ O, float* __restrict__ part, int H,
    int block_size, int max_blocks, int num_blocks, float c) {
  constexpr int LPR = D / 8;                 // lanes per key row (16 bytes each)
  constexpr int RPI = 64 / LPR;              // key rows per load instruction
  constexpr int NL = PG_UNIT / RPI;          // loads per unit and matrix
  constexpr int NSPLIT = PG_NW * RPI;        // partial results per workgroup
  __shared__ float sm[NSPLIT], sl[NSPLIT];
  __shared__ float so[NSPLIT][D];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rgrp = lane / LPR, chunk = lane % LPR;
  const int bh = blockIdx.x, b = bh / H, h = bh % H;

  int len = seq_lens[b];
  const int cap = max_blocks * block_size;
  len = len < 1 ? 1 : (len > cap ? cap : len);           // never trust it further than the table
  const int all_units = (len + PG_UNIT - 1) / PG_UNIT;
  const int upb = block_size / PG_UNIT;                  // units per cache block
  // the units this workgroup takes: all of them, or its range of a cut into gridDim.y ranges of
  // equal length (a multiple of the wavefront count; the last ranges of a short sequence are empty)
  int u_begin = 0, nunits = all_units;
  if (SPLIT) {
    const int nsplit = (int)gridDim.y;
    const int per = ((all_units + nsplit - 1) / nsplit + PG_NW - 1) / PG_NW * PG_NW;
    u_begin = (int)blockIdx.y * per;
    nunits = u_begin + per < all_units ? u_begin + per : all_units;
  }

  // this lane's 8 query elements, as packed pairs
  const u32x4 qv = *reinterpret_cast<const u32x4_mem*>(Q + (int64_t)bh * D + chunk * 8);

  // first element of unit u in the cache (block number clamped: a bad table entry may give a
  // wrong answer but never an access outside the cache)
  auto unit_base = [&](int u) -> int64_t {
    int pb = block_table[(int64_t)b * max_blocks + u / upb];
    pb = pb < 0 ? 0 : (pb >= num_blocks ? num_blocks - 1 : pb);
    return (((int64_t)pb * H + h) * block_size + (u % upb) * PG_UNIT) * D;
  };
  const int lane_off = rgrp * D + chunk * 8;             // + i * RPI * D for load i
  auto load_unit = [&](int u, u32x4 (&kf)[NL], u32x4 (&vf)[NL]) {
    const int64_t base = unit_base(u) + lane_off;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      kf[i] = load_stream16(Kc + base + i * RPI * D);     // the cache is read once: streaming loads
      vf[i] = load_stream16(Vc + base + i * RPI * D);
    }
  };

  float m = -__builtin_inff(), l = 0.f;                  // this row group's running maximum (log2 domain) and sum
  float o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;

  u32x4 kf[2][NL], vf[2][NL];
  if (u_begin + wave < nunits) load_unit(u_begin + wave, kf[0], vf[0]);
  int cur = 0;
  for (int u = u_begin + wave; u < nunits; u += PG_NW) {
    if (u + PG_NW < nunits) {
      if (cur == 0) load_unit(u + PG_NW, kf[1], vf[1]); else load_unit(u + PG_NW, kf[0], vf[0]);
    }
    // scores of this lane's keys of the unit: key position u*16 + i*RPI + rgrp
    float x[NL];
    float mx = m;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const u32x4 k = cur == 0 ? kf[0][i] : kf[1][i];
      float s = Dot2<Tag>::f(qv[0], k[0], 0.f);
      s = Dot2<Tag>::f(qv[1], k[1], s);
      s = Dot2<Tag>::f(qv[2], k[2], s);
      s = Dot2<Tag>::f(qv[3], k[3], s);
      s = row_sum<LPR>(s);
      const int p = u * PG_UNIT + i * RPI + rgrp;
      x[i] = p < len ? s * c : -__builtin_inff();
      mx = __builtin_fmaxf(mx, x[i]);
    }
    if (mx != -__builtin_inff()) {                        // else: nothing visible yet in this group
      const float alpha = __builtin_amdgcn_exp2f(m - mx);  // m = -inf gives 0
      l *= alpha;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] *= alpha;
      m = mx;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const float pw = __builtin_amdgcn_exp2f(x[i] - m);       // exp2(-inf) = 0 for masked keys
        const uint32_t pb16 = Elem<Tag>::from_f32(pw);           // weight rounded to the 16-bit type
        l += Elem<Tag>::to_f32((uint16_t)pb16);
        const uint32_t plo = pb16, phi = pb16 << 16;
        u32x4 v = cur == 0 ? vf[0][i] : vf[1][i];
        // slots past seq_len may hold anything (also NaN, and 0 * NaN is NaN): take zeros instead
        if (u * PG_UNIT + i * RPI + rgrp >= len) v = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          o[2 * w] = Dot2<Tag>::f(v[w], plo, o[2 * w]);           // low element of the pair times p
          o[2 * w + 1] = Dot2<Tag>::f(v[w], phi, o[2 * w + 1]);   // high element times p
        }
      }
    }
    cur ^= 1;
  }

  // ---- all partial results meet in LDS; D threads combine them
  const int sidx = wave * RPI + rgrp;
  if (chunk == 0) { sm[sidx] = m; sl[sidx] = l; }
#pragma unroll
  for (int e = 0; e < 8; ++e) so[sidx][chunk * 8 + e] = o[e];
  __syncthreads();
  if (tid < D) {
    float M = sm[0];
#pragma unroll
    for (int s = 1; s < NSPLIT; ++s) M = __builtin_fmaxf(M, sm[s]);
    // a range past the end of a short sequence saw no key at all: its sum and outputs are zeros
    // (the weights below must not become exp2(-inf - -inf))
    const float Mref = SPLIT && M == -__builtin_inff() ? 0.f : M;
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int s = 0; s < NSPLIT; ++s) {
      const float wgt = __builtin_amdgcn_exp2f(sm[s] - Mref);    // empty groups: exp2(-inf) = 0
      L += sl[s] * wgt;
      acc += so[s][tid] * wgt;
    }
    if (SPLIT) {
      float* out = part + ((int64_t)bh * gridDim.y + blockIdx.y) * (2 + D);
      if (tid == 0) { out[0] = M; out[1] = L; }
      out[2 + tid] = acc;
    } else {
      O[(int64_t)bh * D + tid] = Elem<Tag>::from_f32(acc / L);
    }
  }
}

// One workgroup of D threads per (sequence, head): the ranges' partial results, in index order.
// Range 0 is never empty (a sequence has at least one key), so the maximum is finite.
template <typename Tag, int D>
__global__ __launch_bounds__(D) void paged_merge_kernel(const float* __restrict__ part,
                                                        uint16_t* __restrict__ O, int nsplit) {
  // the ranges' maxima and sums go through LDS (one load each, all in flight together), the
  // output slices are read with eight loads in flight per thread: a plain loop over the ranges
  // would wait for one memory round trip after the other (measured 16 us for 32 ranges)
  __shared__ float sm[64], sl[64];
  const int bh = blockIdx.x, tid = threadIdx.x;
  const float* p = part + (int64_t)bh * nsplit * (2 + D);
  if (tid < nsplit) {
    sm[tid] = p[tid * (2 + D)];
    sl[tid] = p[tid * (2 + D) + 1];
  }
  __syncthreads();
  float M = sm[0];
  for (int s = 1; s < nsplit; ++s) M = __builtin_fmaxf(M, sm[s]);
  float L = 0.f, acc = 0.f;
#pragma unroll 8
  for (int s = 0; s < nsplit; ++s) {
    const float wgt = __builtin_amdgcn_exp2f(sm[s] - M);           // empty ranges: exp2(-inf) = 0
    L += sl[s] * wgt;
    acc += p[s * (2 + D) + 2 + tid] * wgt;
  }
  O[(int64_t)bh * D + tid] = Elem<Tag>::from_f32(acc / L);
}

template <typename Tag, int D>
int launch_paged(const PagedArgs& a, int nsplit, float* part, hipStream_t s) {
  const float c = a.scale * 1.4426950408889634f;
  const unsigned pairs = (unsigned)(a.B * a.H);
  if (nsplit <= 1) {
    hipLaunchKernelGGL((paged_decode_kernel<Tag, D, false>), dim3(pairs), dim3(PG_NT), 0, s,
                       a.Q, a.Kc, a.Vc, a.block_table, a.seq_lens, a.O, (float*)nullptr, (int)a.H,
                       (int)a.block_size, (int)a.max_blocks, (int)a.num_blocks, c);
    return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
  }
  hipLaunchKernelGGL((paged_decode_kernel<Tag, D, true>), dim3(pairs, (unsigned)nsplit), dim3(PG_NT), 0, s,
                     a.Q, a.Kc, a.Vc, a.block_table, a.seq_lens, a.O, part, (int)a.H,
                     (int)a.block_size, (int)a.max_blocks, (int)a.num_blocks, c);
  if (hipGetLastError() != hipSuccess) return MLT_ERR_LAUNCH;
  hipLaunchKernelGGL((paged_merge_kernel<Tag, D>), dim3(pairs), dim3(D), 0, s, part, a.O, nsplit);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

}  // namespace

// Ranges per (sequence, head): 1 while the pairs alone give every CU a workgroup; otherwise what
// brings the launch to two workgroups per CU, as long as a range of the longest possible sequence
// (the table's width) keeps at least 16 units (256 keys), and at most 32 (measured on 8 to 256
// pairs of 2k to 32k keys: more ranges than that lose to their own start and end).
int plan_paged_split(const PagedArgs& a) {
  if (a.forced_split > 0) return a.forced_split > 64 ? 64 : a.forced_split;
  DeviceInfo di;
  const int64_t ncu = device_info(di) ? di.ncu : 256;
  const int64_t pairs = a.B * a.H;
  if (pairs > ncu) return 1;
  const int64_t max_units = (a.max_blocks * a.block_size + PG_UNIT - 1) / PG_UNIT;
  int64_t n = (2 * ncu + pairs - 1) / pairs;
  if (n > max_units / 16) n = max_units / 16;
  if (n > 32) n = 32;
  return n < 1 ? 1 : (int)n;
}

int run_paged_decode(const PagedArgs& a, hipStream_t s, int* nsplit_out) {
  int nsplit = plan_paged_split(a);
  float* part = nullptr;
  if (nsplit > 1) {
    part = cached_scratch(a.B * a.H * nsplit * (2 + a.D) * (int64_t)sizeof(float), s);
    if (!part) nsplit = 1;                               // no scratch to be had: the plain form
  }
  if (nsplit_out) *nsplit_out = nsplit;
  if (a.dtype == MLT_BF16)
    return a.D == 128 ? launch_paged<bf16_tag, 128>(a, nsplit, part, s) : launch_paged<bf16_tag, 64>(a, nsplit, part, s);
  return a.D == 128 ? launch_paged<f16_tag, 128>(a, nsplit, part, s) : launch_paged<f16_tag, 64>(a, nsplit, part, s);
}

}  // namespace mlt
