// Pieces shared by the attention-forward kernels for gfx950 (mha_pp.hip, mha_fr.hip): tile sizes,
// the direct global->LDS load, lane-pair exchanges, the workgroup->item map and the LDS layout of
// a K/V tile (paper: arXiv 2503.14985, Section 2.5, Algorithm 1 and Table 5).
#pragma once

#include "mlt_common.h"

namespace mlt {

constexpr int PA_BM = 256;    // query rows per workgroup
constexpr int PA_BN = 64;     // keys per tile
constexpr int PA_NT = 512;
constexpr int PA_NS = 5;      // LDS ring slots (two-group kernels)
constexpr int PA_AHEAD = 3;   // tiles fetched ahead of the softmax phase that issues the fetch
constexpr float PA_LAZY_T = 8.f;   // log2 units a row maximum may grow before the reference point moves

// max / sum of a per-lane value with the one held by lane l ^ 32 (the other half of the keys of
// the same query): permlane32_swap fed the same register twice returns both halves' values.
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
// O^T accumulators -> 16-byte pieces of O rows. A lane holds, of its query row, 4 consecutive d
// per register group g (d = 32t + 8g + 4h + 0..3, h = lane / 32): 8-byte pieces, which the lane
// with the other h interleaves. Swapping group g+1 of the lower lanes with group g of the upper
// ones (permlane32_swap, per packed register) leaves the lower lane with d = 32t + 8g + 0..7 and
// the upper lane with the next 8: one 16-byte store each instead of two 8-byte ones, and 32
// contiguous bytes per row and store instruction.
template <typename Tag>
__device__ __forceinline__ u32x4 o_piece16(const f32x16& acc, int g, float inv) {
  const uint32_t a0 = Elem<Tag>::pack2(acc[4 * g] * inv, acc[4 * g + 1] * inv);
  const uint32_t a1 = Elem<Tag>::pack2(acc[4 * g + 2] * inv, acc[4 * g + 3] * inv);
  const uint32_t b0 = Elem<Tag>::pack2(acc[4 * g + 4] * inv, acc[4 * g + 5] * inv);
  const uint32_t b1 = Elem<Tag>::pack2(acc[4 * g + 6] * inv, acc[4 * g + 7] * inv);
  auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
  auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
  return u32x4{(uint32_t)s0[0], (uint32_t)s1[0], (uint32_t)s0[1], (uint32_t)s1[1]};
}

__device__ __forceinline__ float max3(float a, float b, float c) {
  return __builtin_fmaxf(__builtin_fmaxf(a, b), c);       // v_max3_f32
}

// Workgroup id -> (batch*head, query tile): every XCD owns a contiguous range of the items, and
// the query tiles of one head are walked last tile first (with the causal mask it has the most
// work). All tiles of a head share one XCD's L2.
__device__ __forceinline__ void block_map(int bid, int total, int nq, int nxcd, int& bh, int& qt) {
  const int logical = logical_block(bid, total, nxcd);
  bh = logical / nq;
  qt = nq - 1 - logical % nq;
}

template <int D> struct PaCfg {
  static constexpr int ROWB = D * 2;               // bytes per key row
  static constexpr int TILE_B = PA_BN * ROWB;      // one K or V tile
  static constexpr int SLOT_B = 2 * TILE_B;        // K tile then V tile
  static constexpr int SMEM = PA_NS * SLOT_B;      // 160 KB (D = 128) / 80 KB (D = 64)
  static constexpr int CPR = D / 8;                // 16-byte chunks per row
  static constexpr int RPB = 64 / CPR;             // rows per 1 KB block (one wavefront load)
  static constexpr int NBLK = PA_BN / RPB;         // blocks per tile
  static constexpr int LPW = NBLK / 8;             // loads per wavefront per tile and matrix
  static constexpr int NKK = D / 16;               // k slices of S^T = K Q^T
  static constexpr int NDT = D / 32;               // 32-row tiles of O^T
  // Swizzles. K rows are read 16 at a time at one chunk position (ds_read_b128), V rows 4 at a
  // time over 4 adjacent chunks (ds_read_b64_tr_b16); each must cover 16 distinct bank groups.
  static __device__ __forceinline__ int fk(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  static __device__ __forceinline__ int fv(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }
};

}  // namespace mlt
