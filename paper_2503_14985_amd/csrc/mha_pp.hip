// Attention forward O = softmax(scale * Q K^T [+ causal mask]) V for gfx950, two-group schedule.
//
// The algorithm is the FlashAttention-2 forward of the paper (arXiv 2503.14985, Section 2.5,
// Algorithm 1): Q is loaded once, K/V tiles stream through the loop, the two products sit back to
// back with an online softmax in between, and the output tile is split over the wavefronts along
// its rows only (the paper's warpsPerCTA = [numWarps, 1]), so no softmax statistic ever crosses a
// wavefront. As the paper's layout table (Table 5) asks, P goes from the first product into the
// second without being redistributed; on CDNA4 that holds when both products are computed
// transposed,
//   S^T = K_j Q^T      MFMA A operand = K_j rows (LDS), B operand = Q^T (registers)
//   O^T += V_j^T P^T   MFMA A operand = V_j^T (LDS, transposing read), B operand = P^T
// because a 32x32 accumulator gives lane l one column (one query) and 16 rows (keys), which is
// exactly what the B operand of the next MFMA wants. Row statistics are per lane: the row maximum
// needs one exchange with lane l^32, the row sum none until the end.
//
// Schedule. Workgroup = 8 wavefronts x 32 query rows; key tile 64. A CU runs one workgroup, two
// wavefronts per SIMD (wavefronts w and w+4). Per key tile j a wavefront alternates between
//   X_j  the softmax of S_j on the vector ALU (exp2, max, sum, conversion to 16 bit), and
//   C_j  32 MFMAs back to back: O^T += V_j^T P_j^T, then S_{j+1}^T = K_{j+1} Q^T,
// and the two wavefronts of a SIMD are kept one phase apart by an extra barrier at the start, so
// that the matrix pipe always has one wavefront feeding it while the other one does the
// exponentials: the two kinds of work overlap instead of queueing behind each other. Every phase
// ends in a workgroup barrier.
//
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4), into a ring of 5
// slots (tile t in slot t % 5), fetched three tiles ahead. The tiles are stored unpadded; bank
// conflicts are avoided by choosing which 16-byte chunk each lane fetches (XOR swizzles, below).
#include <type_traits>

#include "mha_tile.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

// D = 64 needs half the LDS (80 KB), so two workgroups fit a CU when the kernel stays within 128
// registers (4 wavefronts per SIMD); while one workgroup waits at a barrier the other one runs
// (measured +6 %). D = 128 fills the LDS with one workgroup.
template <typename Tag, int D, bool CAUSAL>
__global__ __launch_bounds__(PA_NT, D == 64 ? 4 : 1) void mha_pp_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, uint16_t* __restrict__ O, int Sq, int Sk, int nq, int total,
    int nxcd, float c, int negate) {
  typedef PaCfg<D> L;
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int NKK = L::NKK, NDT = L::NDT, ROWB = L::ROWB;
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                             // waves w and w+4 share a SIMD
  const int lq = lane & 31, h = lane >> 5;
  int bh, qt;
  block_map(blockIdx.x, total, nq, nxcd, bh, qt);
  const int q0 = qt * PA_BM + wave * 32;                 // first query row of this wavefront
  const int my_q = q0 + lq;

  const uint16_t* Qh = Q + (int64_t)bh * Sq * D;
  const char* Kh = reinterpret_cast<const char*>(K + (int64_t)bh * Sk * D);
  const char* Vh = reinterpret_cast<const char*>(V + (int64_t)bh * Sk * D);

  // Keys this workgroup looks at. Causal, top-left aligned: key j is visible to query i iff
  // j <= i, so nothing beyond the last query row of the tile is needed.
  int kv_len = Sk;
  if (CAUSAL) {
    const int last_q = (qt + 1) * PA_BM < Sq ? (qt + 1) * PA_BM : Sq;      // exclusive
    kv_len = last_q < Sk ? last_q : Sk;
  }
  const int nblk = (kv_len + PA_BN - 1) / PA_BN;
  // Causal: this wavefront has visible keys in tiles 0 .. my_nblk-1 only.
  int my_nblk = nblk;
  if (CAUSAL) {
    const int need = (q0 + 31) / PA_BN + 1;
    my_nblk = need < nblk ? need : nblk;
  }

  // ---- Q^T operand, resident in registers: query lq, d = 16*kk + 8*h .. +7. A negative scale is
  // applied as a sign flip of Q (exact), so the softmax below always sees c >= 0.
  V8 qf[NKK];
  {
    const int row = my_q < Sq ? my_q : Sq - 1;
    const uint16_t* qp = Qh + (int64_t)row * D + 8 * h;
    const uint32_t flip = negate ? 0x80008000u : 0u;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      u32x4 raw = *reinterpret_cast<const u32x4_mem*>(qp + kk * 16);
      raw[0] ^= flip; raw[1] ^= flip; raw[2] ^= flip; raw[3] ^= flip;
      qf[kk] = __builtin_bit_cast(V8, raw);
    }
  }

  // ---- global -> LDS assignments: wavefront w fills blocks w*LPW .. of the K tile and of the V
  // tile; lane l owns the 16-byte slot l of a block.
  uint32_t voff_k[L::LPW], voff_v[L::LPW];
  int ld_row[L::LPW];
#pragma unroll
  for (int i = 0; i < L::LPW; ++i) {
    const int row = (wave * L::LPW + i) * L::RPB + lane / L::CPR;
    const int slot = lane % L::CPR;
    ld_row[i] = row;
    voff_k[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fk(row)) * 16u;
    voff_v[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fv(row)) * 16u;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  auto issue_tile = [&](int t) {
    const uint32_t dst = lds0 + (t % PA_NS) * L::SLOT_B + wave * L::LPW * 1024;
    const char* kp = Kh + (int64_t)t * L::TILE_B;
    const char* vp = Vh + (int64_t)t * L::TILE_B;
    if ((t + 1) * PA_BN <= Sk) {
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(kp, voff_k[i], dst + i * 1024);
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(vp, voff_v[i], dst + L::TILE_B + i * 1024);
    } else {
      // ragged last tile: rows past Sk re-read row Sk-1 (their weights are forced to 0)
      const int last = Sk - 1 - t * PA_BN;
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(kp, voff_k[i] - back, dst + i * 1024);
      }
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(vp, voff_v[i] - back, dst + L::TILE_B + i * 1024);
      }
    }
  };

  // ---- fragment addresses inside a slot
  // K rows as MFMA A operand: key row lq of a 32-key sub-tile, chunk 2*kk + h, swizzled; the
  // k slice enters by XOR (kk << 5 touches only chunk bits that 2*kk owns).
  const int k_frag = lq * ROWB + ((h ^ L::fk(lq)) << 4);
  // V^T as MFMA A operand through the transposing read: 16-lane group vg serves output rows
  // d = 16*(vg%2) + i and contraction half vg/2; lane vs of the group addresses key row
  // 4*(vg/2) + vs/4 (+8 for the second read) and d columns 4*(vs%4)..+3. The 32-row tile t of
  // O^T enters by XOR (t << 6).
  const int vg = lane >> 4, vs = lane & 15;
  const int v_row = 4 * (vg >> 1) + (vs >> 2);
  const int v_frag = L::TILE_B + v_row * ROWB + (((2 * (vg & 1) + ((vs & 3) >> 1)) ^ L::fv(v_row)) << 4) + 8 * (vs & 1);

  f32x16 o_acc[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
  f32x16 s_acc[2];
  u32x4 pq[4];                       // P^T of the current tile as MFMA operands: one per 16 keys
  float mc_run = -__builtin_inff();  // running maximum of the scores, times c (log2 domain)
  float l_run = 0.f;                 // running sum over this lane's half of the keys

  // Operand fragments are fetched in chunks of NDT fragments (NDT MFMAs each). A compute phase
  // runs 8 chunks: V_j groups 0..3 (16 keys each), then K_{j+1} chunks 0..3. Two chunk buffers;
  // the fragment that will take a buffer entry next is requested right after the MFMA that read
  // the entry has been issued, so between two MFMAs the wavefront issues at most two LDS reads
  // and one address computation (which the 32 clocks of the running MFMA cover), and every
  // request has about two chunks (2 * NDT MFMAs) of time to arrive.
  V8 fb[2][NDT];
  // Fragment addresses are kept as complete LDS addresses in registers, one per XOR variant (the
  // k slices of K, the 32-row tiles of V^T), and moved from slot to slot by one addition per tile;
  // everything else about a read is an immediate offset. (Recomputing the XOR per read costs a
  // vector ALU instruction per MFMA, and the vector ALU is what this kernel is short of.)
  uint32_t ka[NKK], va[NDT];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) ka[kk] = lds0 + (uint32_t)(k_frag ^ (kk << 5));
#pragma unroll
  for (int t = 0; t < NDT; ++t) va[t] = lds0 + (uint32_t)(v_frag ^ (t << 6));
  auto read_v_frag = [&](int g, int t, V8& f) {
    const uint32_t a = va[t] + g * 16 * ROWB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)a);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)(a + 8 * ROWB));
    f = join_tr<V8>(lo, hi);
  };
  // K fragment fi of a tile: sub-tile fi & 1 (the two S^T accumulators alternate), k slice fi >> 1
  auto read_k_frag = [&](int fi, V8& f) {
    const uint32_t a = ka[fi >> 1] + (fi & 1) * 32 * ROWB;
    f = __builtin_bit_cast(V8, *(const MLT_LDS u32x4*)(uintptr_t)a);
  };
  auto mfma_v = [&](int g, int t, const V8& f) {
    o_acc[t] = mfma32(f, __builtin_bit_cast(V8, pq[g]), o_acc[t]);
  };
  auto mfma_k = [&](int fi, const V8& f) {
    if (fi < 2) {                                         // first slice: start from zero
      f32x16 z;
#pragma unroll
      for (int r = 0; r < 16; ++r) z[r] = 0.f;
      s_acc[fi & 1] = mfma32(f, qf[fi >> 1], z);
    } else {
      s_acc[fi & 1] = mfma32(f, qf[fi >> 1], s_acc[fi & 1]);
    }
  };
#define MLT_SB() __builtin_amdgcn_sched_barrier(0)

  // ---- softmax of S_j (in s_acc) -> pq, mc_run, rescaled o_acc and l_run
  auto softmax_tile = [&](int j) {
    const int kb0 = j * PA_BN;
    // register r of sub-tile kb is key kb0 + 32*kb + 8*(r/4) + 4*h + r%4
    const bool need_mask = (CAUSAL && (kb0 + PA_BN - 1 > q0)) || (kb0 + PA_BN > Sk);
    if (need_mask) {
      // last visible key, relative to the first key this lane holds; a masked score becomes -inf
      // (c > 0 always, see the launcher: its weight is then exactly exp2(-inf) = 0)
      const int limit = CAUSAL ? (my_q < Sk - 1 ? my_q : Sk - 1) : Sk - 1;
      const int rel = limit - (kb0 + 4 * h);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (32 * kb + 8 * (r >> 2) + (r & 3) > rel) s_acc[kb][r] = -__builtin_inff();
    }
    float mx = max3(s_acc[0][0], s_acc[0][1], s_acc[0][2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = max3(mx, s_acc[0][r], s_acc[0][r + 1]);
    mx = max3(mx, s_acc[0][15], s_acc[1][0]);
#pragma unroll
    for (int r = 1; r < 15; r += 2) mx = max3(mx, s_acc[1][r], s_acc[1][r + 1]);
    mx = __builtin_fmaxf(mx, s_acc[1][15]);
    mx = both_halves_max(mx);
    // Lazy rescale: the reference point mc_run only moves when some row's maximum has grown by
    // more than PA_LAZY_T in the log2 domain (weights then stay below 2^8, far inside fp32 and
    // 16-bit range); mathematically the result does not depend on the reference point. The price:
    // the largest weight of a row is no longer exactly 1, so it is rounded to 16 bit like the rest.
    const float t = mx * c;
    const bool grow = t - mc_run > PA_LAZY_T;                    // true on the first tile (mc_run = -inf)
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      const float mc_new = grow ? t : mc_run;
      const float alpha = grow ? __builtin_amdgcn_exp2f(mc_run - t) : 1.f;   // 0 on the first tile
      l_run *= alpha;
#pragma unroll
      for (int tt = 0; tt < NDT; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[tt][r] *= alpha;
      mc_run = mc_new;
    }
    {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r], c, -mc_run));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r + 1], c, -mc_run));
          pq[2 * kb + r / 8][(r / 2) & 3] = Elem<Tag>::pack2(p0, p1);
        }
    }
  };

  // ---- schedule
  // Phase p ends at workgroup barrier p. Group 0: X_j in phase 2j, C_j in phase 2j+1; group 1 one
  // phase later. Tile t is first read (K_t, by C_{t-1} of group 0) in phase 2t-1 and last read
  // (V_t, by C_t of group 1) in phase 2t+2. In X_j every wavefront issues its share of tile j+3
  // into the slot of tile j-2 (last read in phase 2j-2, before both groups' X_j) and then needs
  // its share of tile j+1 complete before group 0's C_j (phase 2j+1) starts:
  //   group 0 waits at the end of X_j (phase 2j) with the shares of tiles j+2, j+3 still in flight,
  //   group 1 waits at the end of C_{j-1} (also phase 2j) with the share of tile j+2 in flight.
  constexpr int LPT = 2 * L::LPW;                         // loads per wavefront per tile
#pragma unroll
  for (int t = 0; t < PA_AHEAD; ++t)
    if (t < nblk) issue_tile(t);
  // tile 0 (and with it K_0) must be complete for everyone: the prologue computes S_0
  if (nblk >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 15));
  else if (nblk == 2) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
  else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
  MLT_BARRIER();
  if (grp == 1) MLT_BARRIER();            // stagger: group 1 runs one phase behind

  // prologue: S_0 = K_0 Q^T, then the first two V_0 groups (a compute phase without the P V part)
  {
    if (my_nblk > 0) {                                    // ka, va point into slot 0
#pragma unroll
      for (int i = 0; i < NDT; ++i) read_k_frag(i, fb[0][i]);
#pragma unroll
      for (int i = 0; i < NDT; ++i) read_k_frag(NDT + i, fb[1][i]);
      MLT_SB();
#pragma unroll
      for (int ch = 0; ch < 4; ++ch)
#pragma unroll
        for (int i = 0; i < NDT; ++i) {
          mfma_k(ch * NDT + i, fb[ch & 1][i]);
          MLT_SB();
          if (ch < 2) read_k_frag((ch + 2) * NDT + i, fb[ch & 1][i]);
          else read_v_frag(ch - 2, i, fb[ch & 1][i]);
          MLT_SB();
        }
    }
    if (grp == 1) {
      if (nblk >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    }
    MLT_BARRIER();
  }

  int slot_off = 0;                                       // byte offset of tile j's slot
  for (int j = 0; j < nblk; ++j) {
    const int slot_off_next = slot_off + L::SLOT_B == L::SMEM ? 0 : slot_off + L::SLOT_B;
    const bool active = j < my_nblk;                       // wavefront-uniform
    const bool active_next = j + 1 < my_nblk;
    // ---- X_j (the first two V_j groups are already in the chunk buffers)
    if (j + PA_AHEAD < nblk) issue_tile(j + PA_AHEAD);
    __builtin_amdgcn_sched_barrier(0);
    if (active) {
      softmax_tile(j);
      // keep the whole softmax on this side of the barrier (the weights are only consumed after it)
#pragma unroll
      for (int g = 0; g < 4; ++g) asm volatile("" : "+v"(pq[g]));
    }
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 0) {
      // in flight, oldest first: tiles j+1, j+2, j+3 (those that exist)
      const int newer = (j + 3 < nblk ? 1 : 0) + (j + 2 < nblk ? 1 : 0);
      if (newer == 2) __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 0));
      else if (newer == 1) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 0));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
    } else {
      __builtin_amdgcn_s_waitcnt(wait_imm(63, 0));
    }
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    // (measured: with D = 128 the MFMA phase gains 3 % from a raised issue priority, D = 64 loses)
    if (D == 128) __builtin_amdgcn_s_setprio(1);
    // ---- C_j: O^T += V_j^T P_j^T, then S_{j+1}^T = K_{j+1} Q^T, then the first two groups of
    // V_{j+1} into the buffers for the next compute phase. Chunk n's MFMAs alternate with the
    // reads of chunk n+2: V_j groups 2, 3, then K_{j+1} chunks 0..3, then V_{j+1} groups 0, 1.
    // On the way the fragment addresses move on to the slot of tile j+1: ka before the first K
    // read, va after the last V_j read.
    if (active) {
      const uint32_t dslot = (uint32_t)(slot_off_next - slot_off);
      // (on a wavefront's last tile the K reads below fetch fragments nobody uses: cheaper than a
      // branch per MFMA, and the addresses stay inside the ring)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int t = 0; t < NDT; ++t) {
          mfma_v(g, t, fb[g & 1][t]);
          MLT_SB();
          if (g < 2) read_v_frag(g + 2, t, fb[g & 1][t]);
          else read_k_frag((g - 2) * NDT + t, fb[g & 1][t]);
          if (g == 0) { ka[2 * t] += dslot; ka[2 * t + 1] += dslot; }
          if (g == 3) va[t] += dslot;
          MLT_SB();
        }
      if (active_next) {
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
          for (int i = 0; i < NDT; ++i) {
            mfma_k(ch * NDT + i, fb[ch & 1][i]);
            MLT_SB();
            if (ch < 2) read_k_frag((ch + 2) * NDT + i, fb[ch & 1][i]);
            else read_v_frag(ch - 2, i, fb[ch & 1][i]);
            MLT_SB();
          }
      }
      // The row sum of the ROUNDED weights (what P V used) is taken here, behind the last MFMA,
      // while the matrix pipe drains. Measured alternatives: in the softmax phase -5 %; one
      // addition after each P V MFMA -9 % (dot instructions between MFMAs hold the MFMAs up).
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) l_run = Elem<Tag>::add_pair(pq[g][e], l_run);
      asm volatile("" : "+v"(l_run));
    }
    if (D == 128) __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 1) {
      // end of C_j = phase 2j+2 = the phase of group 0's X_{j+1}: tile j+2 must be complete;
      // in flight behind it: tile j+3 (issued in X_j), if it exists
      if (j + 3 < nblk) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    }
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    slot_off = slot_off_next;
  }
#undef MLT_SB
  if (grp == 0) MLT_BARRIER();            // same barrier count for both groups

  // ---- epilogue: O = O^T / l, l summed over both key halves; 8 consecutive d per lane and piece
  const float l_tot = both_halves_sum(l_run);
  const float inv = 1.f / l_tot;
  u32x4 ow[NDT][2];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) ow[t][gp] = o_piece16<Tag>(o_acc[t], 2 * gp, inv);
  // Through LDS (the ring is free: every wavefront is past its last tile read after the barrier
  // above), so that a store instruction writes whole rows: the wavefront parks its 32 rows in its
  // own 32 * ROWB bytes, 16-byte chunk ch of row r at position ch ^ (r % chunks per row), and
  // reads them back 64 / chunks-per-row rows at a time, 1 KB contiguous in O per store. Only the
  // wavefront's own data is involved, and LDS serves a wavefront's accesses in order: no barrier.
  const uint32_t o_lds = lds0 + wave * 32 * ROWB;
  constexpr int CM = L::CPR - 1;
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {
      const int ch = 4 * t + 2 * gp + h;
      *(MLT_LDS u32x4*)(uintptr_t)(o_lds + lq * ROWB + ((ch ^ (lq & CM)) << 4)) = ow[t][gp];
    }
  uint16_t* ob = O + ((int64_t)bh * Sq + q0) * D;
#pragma unroll
  for (int i = 0; i < 32 / L::RPB; ++i) {
    const int r = i * L::RPB + lane / L::CPR, cc = lane % L::CPR;
    const u32x4 v = *(const MLT_LDS u32x4*)(uintptr_t)(o_lds + r * ROWB + ((cc ^ (r & CM)) << 4));
    if (q0 + r < Sq) *reinterpret_cast<u32x4_mem*>(ob + (int64_t)r * D + cc * 8) = v;
  }
}


// ---------------------------------------------------------------------------------------------
// Persistent form of the kernel above for the unmasked case. A workgroup that handles one
// (batch*head, query tile) item and exits pays, per item, for its launch, the latency of the Q
// load, the latency of the first K/V tiles, the one-phase stagger of the two groups at both ends
// and the draining of the O stores: about 10 us per item for D = 128, against 1.7 us per key tile.
// Here the grid is one workgroup per CU and each workgroup walks through items
// blockIdx.x, blockIdx.x + gridDim.x, ... as ONE stream of K/V tiles: the ring of LDS slots, the
// prefetch distance and the phase structure run on across item boundaries, so the first tiles of
// the next item are already in LDS when the current item ends. At a boundary
//   - the softmax phase of an item's LAST tile also issues the loads of the next item's Q operand
//     into the Q registers (they are dead from there on: S of the last tile has been computed),
//   - the compute phase of that tile ends with S_0 of the NEXT item instead of S_{j+1},
//   - the softmax phase of the next item's FIRST tile starts by normalising and storing the
//     finished O tile and clearing the accumulators.
// Only the first and the last item of a workgroup see a prologue, a stagger phase and a drain.
//
// Counting vector memory operations: besides the K/V loads the in-order queue that s_waitcnt
// vmcnt looks at now also holds the Q loads and the O stores. An s_waitcnt vmcnt(N) is correct as
// long as N does not exceed the number of operations issued after the one that is needed, so the
// waits below add the Q loads / O stores to N only where they are certain to have been issued (a
// wavefront whose query rows all lie beyond Sq issues no stores and adds nothing).
template <typename Tag, int D>
__global__ __launch_bounds__(PA_NT, 1) void mha_ps_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, uint16_t* __restrict__ O, int Sq, int Sk, int nq, int total,
    int nxcd, float c, int negate) {
  typedef PaCfg<D> L;
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int NKK = L::NKK, NDT = L::NDT, ROWB = L::ROWB;
  constexpr int LPT = 2 * L::LPW;    // K/V loads per wavefront per tile
  constexpr int NQL = NKK;           // loads per wavefront that fetch a Q operand
  constexpr int NST = 2 * NDT;       // stores per wavefront that write an O tile
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                             // waves w and w+4 share a SIMD
  const int lq = lane & 31, h = lane >> 5;
  const int G = (int)gridDim.x;
  const int nblk = (Sk + PA_BN - 1) / PA_BN;             // key tiles per item, >= 2 (launcher)
  const int n_items = (total - (int)blockIdx.x + G - 1) / G;   // >= 1 (launcher: G <= total)
  const int NT = n_items * nblk;                         // tiles in this workgroup's stream

  const char* Kb = reinterpret_cast<const char*>(K);
  const char* Vb = reinterpret_cast<const char*>(V);
  const int64_t head_b = (int64_t)Sk * ROWB;             // bytes of one head's K (or V)

  // ---- Q^T operand of an item: query lq of the wavefront's 32 rows, d = 16*kk + 8*h .. +7.
  // Loaded by inline assembly, so that the compiler does not track the loads: inside the loop it
  // could only wait for them in every iteration, K/V loads included. q_issue starts the loads;
  // the registers hold the operand only after the schedule's own wait and q_finish (which also
  // applies a negative scale as a sign flip, so the softmax always sees c >= 0).
  u32x4 qf[NKK];
  const uint32_t flip = negate ? 0x80008000u : 0u;
  auto q_issue = [&](int bh_, int q0_) __attribute__((always_inline)) {
    const int my_q_ = q0_ + lq;
    const int row = my_q_ < Sq ? my_q_ : Sq - 1;
    const uint16_t* qp = Q + ((int64_t)bh_ * Sq + row) * D + 8 * h;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(qf[kk]) : "v"(qp + kk * 16) : "memory");
  };
  auto q_finish = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      asm volatile("" : "+v"(qf[kk]));
      qf[kk][0] ^= flip; qf[kk][1] ^= flip; qf[kk][2] ^= flip; qf[kk][3] ^= flip;
    }
  };

  // ---- global -> LDS: wavefront w fills blocks w*LPW .. of the K tile and of the V tile; lane l
  // owns the 16-byte slot l of a block.
  uint32_t voff_k[L::LPW], voff_v[L::LPW];
  int ld_row[L::LPW];
#pragma unroll
  for (int i = 0; i < L::LPW; ++i) {
    const int row = (wave * L::LPW + i) * L::RPB + lane / L::CPR;
    const int slot = lane % L::CPR;
    ld_row[i] = row;
    voff_k[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fk(row)) * 16u;
    voff_v[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fv(row)) * 16u;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  // The prefetch cursor: stream tile pf_g = tile pf_j of item pf_item, goes to ring offset pf_slot.
  int pf_g = 0, pf_j = 0, pf_item = (int)blockIdx.x, pf_slot = 0;
  const char *pf_k, *pf_v;
  {
    int b0, t0;
    block_map(pf_item, total, nq, nxcd, b0, t0);
    pf_k = Kb + (int64_t)b0 * head_b;
    pf_v = Vb + (int64_t)b0 * head_b;
  }
  auto issue_next = [&]() __attribute__((always_inline)) {
    if (pf_g >= NT) return;
    const uint32_t dst = lds0 + pf_slot + wave * L::LPW * 1024;
    const char* kp = pf_k + (int64_t)pf_j * L::TILE_B;
    const char* vp = pf_v + (int64_t)pf_j * L::TILE_B;
    if ((pf_j + 1) * PA_BN <= Sk) {
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(kp, voff_k[i], dst + i * 1024);
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(vp, voff_v[i], dst + L::TILE_B + i * 1024);
    } else {
      // ragged last tile: rows past Sk re-read row Sk-1 (their weights are forced to 0)
      const int last = Sk - 1 - pf_j * PA_BN;
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(kp, voff_k[i] - back, dst + i * 1024);
      }
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(vp, voff_v[i] - back, dst + L::TILE_B + i * 1024);
      }
    }
    ++pf_g;
    pf_slot = pf_slot + L::SLOT_B == L::SMEM ? 0 : pf_slot + L::SLOT_B;
    if (++pf_j == nblk) {
      pf_j = 0;
      pf_item += G;
      if (pf_item < total) {
        int b2, t2;
        block_map(pf_item, total, nq, nxcd, b2, t2);
        pf_k = Kb + (int64_t)b2 * head_b;
        pf_v = Vb + (int64_t)b2 * head_b;
      }
    }
  };

  // ---- fragment addresses (as in mha_pp_kernel)
  const int k_frag = lq * ROWB + ((h ^ L::fk(lq)) << 4);
  const int vg = lane >> 4, vs = lane & 15;
  const int v_row = 4 * (vg >> 1) + (vs >> 2);
  const int v_frag = L::TILE_B + v_row * ROWB + (((2 * (vg & 1) + ((vs & 3) >> 1)) ^ L::fv(v_row)) << 4) + 8 * (vs & 1);

  f32x16 o_acc[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
  f32x16 s_acc[2];
  u32x4 pq[4];
  float mc_run = -__builtin_inff();
  float l_run = 0.f;

  V8 fb[2][NDT];
  uint32_t ka[NKK], va[NDT];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) ka[kk] = lds0 + (uint32_t)(k_frag ^ (kk << 5));
#pragma unroll
  for (int t = 0; t < NDT; ++t) va[t] = lds0 + (uint32_t)(v_frag ^ (t << 6));
  auto read_v_frag = [&](int g, int t, V8& f) __attribute__((always_inline)) {
    const uint32_t a = va[t] + g * 16 * ROWB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)a);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)(a + 8 * ROWB));
    f = join_tr<V8>(lo, hi);
  };
  auto read_k_frag = [&](int fi, V8& f) __attribute__((always_inline)) {
    const uint32_t a = ka[fi >> 1] + (fi & 1) * 32 * ROWB;
    f = __builtin_bit_cast(V8, *(const MLT_LDS u32x4*)(uintptr_t)a);
  };
  auto mfma_v = [&](int g, int t, const V8& f) __attribute__((always_inline)) {
    o_acc[t] = mfma32(f, __builtin_bit_cast(V8, pq[g]), o_acc[t]);
  };
  auto mfma_k = [&](int fi, const V8& f) __attribute__((always_inline)) {
    if (fi < 2) {
      f32x16 z;
#pragma unroll
      for (int r = 0; r < 16; ++r) z[r] = 0.f;
      s_acc[fi & 1] = mfma32(f, __builtin_bit_cast(V8, qf[fi >> 1]), z);
    } else {
      s_acc[fi & 1] = mfma32(f, __builtin_bit_cast(V8, qf[fi >> 1]), s_acc[fi & 1]);
    }
  };
#define MLT_SB() __builtin_amdgcn_sched_barrier(0)

  // ---- softmax of S_j (in s_acc) -> pq, mc_run, rescaled o_acc and l_run (mha_pp_kernel's, without
  // the causal part)
  auto softmax_tile = [&](int j) __attribute__((always_inline)) {
    const int kb0 = j * PA_BN;
    if (kb0 + PA_BN > Sk) {
      const int rel = Sk - 1 - (kb0 + 4 * h);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (32 * kb + 8 * (r >> 2) + (r & 3) > rel) s_acc[kb][r] = -__builtin_inff();
    }
    float mx = max3(s_acc[0][0], s_acc[0][1], s_acc[0][2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = max3(mx, s_acc[0][r], s_acc[0][r + 1]);
    mx = max3(mx, s_acc[0][15], s_acc[1][0]);
#pragma unroll
    for (int r = 1; r < 15; r += 2) mx = max3(mx, s_acc[1][r], s_acc[1][r + 1]);
    mx = __builtin_fmaxf(mx, s_acc[1][15]);
    mx = both_halves_max(mx);
    const float t = mx * c;
    const bool grow = t - mc_run > PA_LAZY_T;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      const float mc_new = grow ? t : mc_run;
      const float alpha = grow ? __builtin_amdgcn_exp2f(mc_run - t) : 1.f;
      l_run *= alpha;
#pragma unroll
      for (int tt = 0; tt < NDT; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[tt][r] *= alpha;
      mc_run = mc_new;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r], c, -mc_run));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][r + 1], c, -mc_run));
        pq[2 * kb + r / 8][(r / 2) & 3] = Elem<Tag>::pack2(p0, p1);
      }
  };

  // ---- O = O^T / l for the item whose accumulators are complete, then a clean start for the next
  auto store_item = [&](int bh_, int q0_) __attribute__((always_inline)) {
    const int my_q_ = q0_ + lq;
    const float l_tot = both_halves_sum(l_run);
    const float inv = 1.f / l_tot;
    u32x4 ow[NDT][2];
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int gp = 0; gp < 2; ++gp) ow[t][gp] = o_piece16<Tag>(o_acc[t], 2 * gp, inv);
    if (my_q_ < Sq) {
      uint16_t* op = O + ((int64_t)bh_ * Sq + my_q_) * D + 8 * h;
#pragma unroll
      for (int t = 0; t < NDT; ++t)
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) *reinterpret_cast<u32x4_mem*>(op + t * 32 + 16 * gp) = ow[t][gp];
    }
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[t][r] = 0.f;
    l_run = 0.f;
    mc_run = -__builtin_inff();
  };

  // s_waitcnt vmcnt(n) lgkmcnt(LG) for a wavefront-uniform n from the set the schedule produces
  // (multiples of LPT plus NQL or NST); anything else waits for everything.
  auto wait_vm0 = [&](int n) __attribute__((always_inline)) {     // with lgkmcnt(0)
    switch (n) {
#define MLT_W(N) case N: __builtin_amdgcn_s_waitcnt(wait_imm(N, 0)); break;
      MLT_W(2) MLT_W(4) MLT_W(6) MLT_W(8) MLT_W(10) MLT_W(12) MLT_W(14) MLT_W(16) MLT_W(18) MLT_W(20) MLT_W(22) MLT_W(24) MLT_W(26) MLT_W(28) MLT_W(30) MLT_W(32)
#undef MLT_W
      default: __builtin_amdgcn_s_waitcnt(wait_imm(0, 0)); break;
    }
  };
  auto wait_vm15 = [&](int n) __attribute__((always_inline)) {    // LDS counter left alone
    switch (n) {
#define MLT_W(N) case N: __builtin_amdgcn_s_waitcnt(wait_imm(N, 15)); break;
      MLT_W(2) MLT_W(4) MLT_W(6) MLT_W(8) MLT_W(10) MLT_W(12) MLT_W(14) MLT_W(16) MLT_W(18) MLT_W(20) MLT_W(22) MLT_W(24) MLT_W(26) MLT_W(28) MLT_W(30) MLT_W(32)
#undef MLT_W
      default: __builtin_amdgcn_s_waitcnt(wait_imm(0, 15)); break;
    }
  };

  // ---- start of the stream: Q of the first item, the first tiles, S_0 (as in mha_pp_kernel)
  int item = (int)blockIdx.x;                 // the item being computed
  int bh, qt;
  block_map(item, total, nq, nxcd, bh, qt);
  int q0 = qt * PA_BM + wave * 32;
  int o_bh = bh, o_q0 = q0;                   // the item the accumulators belong to
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) qf[kk] = u32x4{0u, 0u, 0u, 0u};
  q_issue(bh, q0);
#pragma unroll
  for (int t = 0; t < PA_AHEAD; ++t) issue_next();
  if (NT >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 15));
  else __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));     // NT >= 2
  MLT_BARRIER();
  if (grp == 1) MLT_BARRIER();            // stagger: group 1 runs one phase behind
  q_finish();
  {
#pragma unroll
    for (int i = 0; i < NDT; ++i) read_k_frag(i, fb[0][i]);
#pragma unroll
    for (int i = 0; i < NDT; ++i) read_k_frag(NDT + i, fb[1][i]);
    MLT_SB();
#pragma unroll
    for (int ch = 0; ch < 4; ++ch)
#pragma unroll
      for (int i = 0; i < NDT; ++i) {
        mfma_k(ch * NDT + i, fb[ch & 1][i]);
        MLT_SB();
        if (ch < 2) read_k_frag((ch + 2) * NDT + i, fb[ch & 1][i]);
        else read_v_frag(ch - 2, i, fb[ch & 1][i]);
        MLT_SB();
      }
    if (grp == 1) {
      if (NT >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    }
    MLT_BARRIER();
  }

  // ---- the stream of key tiles: softmax phase X, compute phase C per tile. j is the tile's number
  // inside its item, g its number in the stream.
  int slot_off = 0;           // ring offset of the current tile's slot
  int st_age = 8;             // tiles since this wavefront last issued O stores (0: in this tile)
  int j = 0;
  for (int g = 0; g < NT; ++g) {
    const int slot_off_next = slot_off + L::SLOT_B == L::SMEM ? 0 : slot_off + L::SLOT_B;
    const bool more = g + 1 < NT;                        // S of stream tile g+1 is wanted
    const bool first = j == 0 && g > 0;                  // an item ended with the previous tile
    const bool last = j == nblk - 1 && more;             // another item follows this tile
    // ---- X: Q of the next item (at an item's last tile), stream tile g+3 into the slot of tile
    // g-2, the finished O tile (at an item's first tile), then the softmax of S_g
    if (last) {
      item += G;
      block_map(item, total, nq, nxcd, bh, qt);
      q0 = qt * PA_BM + wave * 32;
      q_issue(bh, q0);
    }
    issue_next();
    MLT_SB();
    if (first) {
      if (o_q0 < Sq) st_age = 0;       // some lane of this wavefront has a row to store
      store_item(o_bh, o_q0);
      o_bh = bh; o_q0 = q0;
    }
    MLT_SB();
    softmax_tile(j);
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(pq[i]));
    MLT_SB();
    if (grp == 0) {
      // needed: tile g+1. Issued after it: tiles g+2, g+3 (those that exist), the O stores of this
      // or the last two tiles' softmax phases, this phase's Q loads.
      if (g + 3 < NT && st_age > 2 && !last) {             // the steady state: one test, one wait
        __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 0));
      } else {
        int n = ((g + 3 < NT ? 1 : 0) + (g + 2 < NT ? 1 : 0)) * LPT;
        if (st_age <= 2) n += NST;
        if (last) n += NQL;
        wait_vm0(n);
      }
    } else {
      __builtin_amdgcn_s_waitcnt(wait_imm(63, 0));
    }
    MLT_BARRIER();
    MLT_SB();
    if (D == 128) __builtin_amdgcn_s_setprio(1);
    // ---- C: O^T += V_g^T P_g^T, then S^T of stream tile g+1 (after the last tile of an item that
    // is K_0 of the next item against the next item's Q), then the first two V groups of tile g+1
    {
      const uint32_t dslot = (uint32_t)(slot_off_next - slot_off);
#pragma unroll
      for (int gi = 0; gi < 4; ++gi)
#pragma unroll
        for (int t = 0; t < NDT; ++t) {
          mfma_v(gi, t, fb[gi & 1][t]);
          MLT_SB();
          if (gi < 2) read_v_frag(gi + 2, t, fb[gi & 1][t]);
          else read_k_frag((gi - 2) * NDT + t, fb[gi & 1][t]);
          if (gi == 0) { ka[2 * t] += dslot; ka[2 * t + 1] += dslot; }
          if (gi == 3) va[t] += dslot;
          MLT_SB();
        }
      if (last) {
        // the Q loads were issued before stream tile g+3 (if there is one)
        if (g + 3 < NT) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
        else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
        q_finish();
        MLT_SB();
      }
      if (more) {
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
          for (int i = 0; i < NDT; ++i) {
            mfma_k(ch * NDT + i, fb[ch & 1][i]);
            MLT_SB();
            if (ch < 2) read_k_frag((ch + 2) * NDT + i, fb[ch & 1][i]);
            else read_v_frag(ch - 2, i, fb[ch & 1][i]);
            MLT_SB();
          }
      }
#pragma unroll
      for (int gi = 0; gi < 4; ++gi)
#pragma unroll
        for (int e = 0; e < 4; ++e) l_run = Elem<Tag>::add_pair(pq[gi][e], l_run);
      asm volatile("" : "+v"(l_run));
    }
    if (D == 128) __builtin_amdgcn_s_setprio(0);
    MLT_SB();
    if (grp == 1) {
      // needed: tile g+2. Issued after it: tile g+3 (if it exists) and the O stores of this tile's
      // or the previous tile's softmax phase.
      if (g + 3 < NT && st_age > 1) {
        __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      } else {
        int n = g + 3 < NT ? LPT : 0;
        if (st_age <= 1) n += NST;
        wait_vm15(n);
      }
    }
    MLT_BARRIER();
    MLT_SB();
    slot_off = slot_off_next;
    ++st_age;
    j = j + 1 == nblk ? 0 : j + 1;
  }
#undef MLT_SB
  if (grp == 0) MLT_BARRIER();            // same barrier count for both groups
  store_item(o_bh, o_q0);
}

// ---------------------------------------------------------------------------------------------
// The same kernel on 16x16x32 MFMAs. Schedule, LDS ring, swizzles, loads and softmax are those of
// mha_pp_kernel above; what changes is the shape of the hardware dot and with it who holds what.
// Measured on N(0,1) operands the chip sustains 2100 TFLOP/s of 16x16x32 bf16 MFMAs against 1850
// TFLOP/s of 32x32x16 (a register-only loop; the chip is power-limited and this shape reads and
// writes half as many accumulator registers per flop), with the same LDS bytes per flop.
//   S^T tile (kt, qt) = K rows 16*kt.. x queries 16*qt..:  lane l holds query l%16 of the q tile
//     and keys 16*kt + 4*(l/16) + r, r = 0..3 (one f32x4); 4 key tiles x 2 query tiles per wavefront;
//   P^T as B operand of O^T += V^T P^T over a 32-key slice ks: a lane's 8 contraction slots are its
//     own 4 + 4 values of the key tiles 2*ks and 2*ks+1, i.e. keys 32*ks + 4*(l/16) + e and
//     32*ks + 16 + 4*(l/16) + e. The contraction order inside a slice is free as long as V^T uses
//     the same one: the two transposing reads of a V^T fragment fetch exactly those two groups of
//     four key rows. Again no data movement between the two products;
//   O^T tile (dt, qt) = d rows 16*dt.. x queries 16*qt..: lane holds d = 16*dt + 4*(l/16) + r;
//   a row's statistics live in the 4 lanes l%16 + 16*g: the row maximum takes two lane swaps
//     (rows of 16, then halves of 32), the row sum none until the end.
__device__ __forceinline__ float four_groups_max(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float m1 = __builtin_fmaxf(__builtin_bit_cast(float, (unsigned)a[0]), __builtin_bit_cast(float, (unsigned)a[1]));
  return both_halves_max(m1);
}
__device__ __forceinline__ float four_groups_sum(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float s1 = __builtin_bit_cast(float, (unsigned)a[0]) + __builtin_bit_cast(float, (unsigned)a[1]);
  return both_halves_sum(s1);
}

template <typename Tag, int D, bool CAUSAL>
__global__ __launch_bounds__(PA_NT, D == 64 ? 4 : 1) void mha_pp16_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, uint16_t* __restrict__ O, int Sq, int Sk, int nq, int total,
    int nxcd, float c, int negate) {
  typedef PaCfg<D> L;
  typedef typename Elem<Tag>::vec8 V8;
  constexpr int NDS = D / 32;                            // 32-deep d slices of S^T = K Q^T
  constexpr int NDT = L::NDT;                            // pairs of 16-row d tiles of O^T (= D / 32)
  constexpr int ROWB = L::ROWB;
  extern __shared__ __align__(16) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                             // waves w and w+4 share a SIMD
  const int l16 = lane & 15, g4 = lane >> 4;
  int bh, qt_wg;
  block_map(blockIdx.x, total, nq, nxcd, bh, qt_wg);
  const int q0 = qt_wg * PA_BM + wave * 32;              // first query row of this wavefront
  int my_q[2];
  my_q[0] = q0 + l16;
  my_q[1] = q0 + 16 + l16;

  const uint16_t* Qh = Q + (int64_t)bh * Sq * D;
  const char* Kh = reinterpret_cast<const char*>(K + (int64_t)bh * Sk * D);
  const char* Vh = reinterpret_cast<const char*>(V + (int64_t)bh * Sk * D);

  int kv_len = Sk;
  if (CAUSAL) {
    const int last_q = (qt_wg + 1) * PA_BM < Sq ? (qt_wg + 1) * PA_BM : Sq;      // exclusive
    kv_len = last_q < Sk ? last_q : Sk;
  }
  const int nblk = (kv_len + PA_BN - 1) / PA_BN;
  int my_nblk = nblk;
  if (CAUSAL) {
    const int need = (q0 + 31) / PA_BN + 1;
    my_nblk = need < nblk ? need : nblk;
  }

  // ---- Q^T operand, resident in registers: query tile qt, d slice ds: query l16, d = 32*ds + 8*g4..
  V8 qf[2][NDS];
  {
    const uint32_t flip = negate ? 0x80008000u : 0u;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      const int row = my_q[qt] < Sq ? my_q[qt] : Sq - 1;
      const uint16_t* qp = Qh + (int64_t)row * D + 8 * g4;
#pragma unroll
      for (int ds = 0; ds < NDS; ++ds) {
        u32x4 raw = *reinterpret_cast<const u32x4_mem*>(qp + ds * 32);
        raw[0] ^= flip; raw[1] ^= flip; raw[2] ^= flip; raw[3] ^= flip;
        qf[qt][ds] = __builtin_bit_cast(V8, raw);
      }
    }
  }

  // ---- global -> LDS assignments (as in mha_pp_kernel)
  uint32_t voff_k[L::LPW], voff_v[L::LPW];
  int ld_row[L::LPW];
#pragma unroll
  for (int i = 0; i < L::LPW; ++i) {
    const int row = (wave * L::LPW + i) * L::RPB + lane / L::CPR;
    const int slot = lane % L::CPR;
    ld_row[i] = row;
    voff_k[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fk(row)) * 16u;
    voff_v[i] = (uint32_t)row * ROWB + (uint32_t)(slot ^ L::fv(row)) * 16u;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  auto issue_tile = [&](int t) {
    const uint32_t dst = lds0 + (t % PA_NS) * L::SLOT_B + wave * L::LPW * 1024;
    const char* kp = Kh + (int64_t)t * L::TILE_B;
    const char* vp = Vh + (int64_t)t * L::TILE_B;
    if ((t + 1) * PA_BN <= Sk) {
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(kp, voff_k[i], dst + i * 1024);
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) load_lds16(vp, voff_v[i], dst + L::TILE_B + i * 1024);
    } else {
      const int last = Sk - 1 - t * PA_BN;
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(kp, voff_k[i] - back, dst + i * 1024);
      }
#pragma unroll
      for (int i = 0; i < L::LPW; ++i) {
        const int back = ld_row[i] > last ? (ld_row[i] - last) * ROWB : 0;
        load_lds16(vp, voff_v[i] - back, dst + L::TILE_B + i * 1024);
      }
    }
  };

  // ---- fragment addresses (complete LDS addresses of slot 0, advanced by one add per tile)
  // K rows as A operand: key row l16 of a 16-key tile (the tile is an immediate), 16-byte chunk
  // 4*ds + g4 of the row, swizzled with the row's key (which the tile offset does not change).
  uint32_t ka[NDS], va[NDT];
#pragma unroll
  for (int ds = 0; ds < NDS; ++ds)
    ka[ds] = lds0 + (uint32_t)(l16 * ROWB + (((4 * ds + g4) ^ L::fk(l16)) << 4));
  // V^T as A operand through the transposing read: lane s = l16 of its 16-lane group addresses
  // key row 4*g4 + s/4 of the slice's first key tile (+ 16 rows for the second read) and the d
  // columns 4*(s%4)..+3 of a 16-wide d tile; d tile dt = 2*t + u: chunk 4*t + 2*u + (s%4)/2, whose
  // 4*t part goes through the swizzle (va[t]) and whose 2*u part is an immediate of 32 bytes.
  {
    const int vrow = 4 * g4 + (l16 >> 2);
    const int c4 = l16 & 3;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
      va[t] = lds0 + (uint32_t)(L::TILE_B + vrow * ROWB + ((((4 * t) ^ L::fv(vrow)) + (c4 >> 1)) << 4) + 8 * (c4 & 1));
  }
  // V fragment (ks, dt): key slice ks (32 keys), d tile dt
  auto read_v_frag = [&](int ks, int dt, V8& f) {
    const uint32_t a = va[dt >> 1] + (dt & 1) * 32 + ks * 32 * ROWB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)a);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLT_LDS s16x4*)(uintptr_t)(a + 16 * ROWB));
    f = join_tr<V8>(lo, hi);
  };
  // K fragment (kt, ds): key tile kt (16 keys), d slice ds
  auto read_k_frag = [&](int kt, int ds, V8& f) {
    f = __builtin_bit_cast(V8, *(const MLT_LDS u32x4*)(uintptr_t)(ka[ds] + kt * 16 * ROWB));
  };

  f32x4 o_acc[2 * NDT][2];                               // [d tile][query tile]
#pragma unroll
  for (int dt = 0; dt < 2 * NDT; ++dt)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) o_acc[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 s_acc[4][2];                                     // [key tile][query tile]
  u32x4 pq[2][2];                                        // P^T operands [key slice][query tile]
  float mc_run[2] = {-__builtin_inff(), -__builtin_inff()};   // per query tile: this lane's query
  float l_run[2] = {0.f, 0.f};

  // Fragments come in chunks of NDT; every fragment feeds two MFMAs (the two query tiles).
  // V chunk cg (0..3): key slice cg / 2, d tiles (cg % 2) * NDT + t; K chunk ch (0..3): key tile ch,
  // d slices 0..NDT-1 (NDS = NDT).
  V8 fb[2][NDT];
  auto read_v_chunk_frag = [&](int cg, int t, V8& f) { read_v_frag(cg >> 1, (cg & 1) * NDT + t, f); };
  auto mfma_v = [&](int cg, int t, const V8& f) {
    const int ks = cg >> 1, dt = (cg & 1) * NDT + t;
    o_acc[dt][0] = mfma16(f, __builtin_bit_cast(V8, pq[ks][0]), o_acc[dt][0]);
    o_acc[dt][1] = mfma16(f, __builtin_bit_cast(V8, pq[ks][1]), o_acc[dt][1]);
  };
  auto mfma_k = [&](int kt, int ds, const V8& f) {
    if (ds == 0) {                                        // first slice: start from zero
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
      s_acc[kt][0] = mfma16(f, qf[0][0], z);
      s_acc[kt][1] = mfma16(f, qf[1][0], z);
    } else {
      s_acc[kt][0] = mfma16(f, qf[0][ds], s_acc[kt][0]);
      s_acc[kt][1] = mfma16(f, qf[1][ds], s_acc[kt][1]);
    }
  };
#define MLT_SB() __builtin_amdgcn_sched_barrier(0)

  // ---- softmax of S_j (in s_acc) -> pq, mc_run, rescaled o_acc and l_run
  auto softmax_tile = [&](int j) {
    const int kb0 = j * PA_BN;
    // register r of tile (kt, qt) is key kb0 + 16*kt + 4*g4 + r for query my_q[qt]
    const bool need_mask = (CAUSAL && (kb0 + PA_BN - 1 > q0)) || (kb0 + PA_BN > Sk);
    if (need_mask) {
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const int limit = CAUSAL ? (my_q[qt] < Sk - 1 ? my_q[qt] : Sk - 1) : Sk - 1;
        const int rel = limit - (kb0 + 4 * g4);
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (16 * kt + r > rel) s_acc[kt][qt][r] = -__builtin_inff();
      }
    }
    float t2[2];
    bool grow[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      float mx = max3(s_acc[0][qt][0], s_acc[0][qt][1], s_acc[0][qt][2]);
      mx = max3(mx, s_acc[0][qt][3], s_acc[1][qt][0]);
      mx = max3(mx, s_acc[1][qt][1], s_acc[1][qt][2]);
      mx = max3(mx, s_acc[1][qt][3], s_acc[2][qt][0]);
      mx = max3(mx, s_acc[2][qt][1], s_acc[2][qt][2]);
      mx = max3(mx, s_acc[2][qt][3], s_acc[3][qt][0]);
      mx = max3(mx, s_acc[3][qt][1], s_acc[3][qt][2]);
      mx = __builtin_fmaxf(mx, s_acc[3][qt][3]);
      mx = four_groups_max(mx);
      t2[qt] = mx * c;
      grow[qt] = t2[qt] - mc_run[qt] > PA_LAZY_T;         // true on the first tile (mc_run = -inf)
    }
    // lazy rescale, as in mha_pp_kernel
    if (__builtin_amdgcn_ballot_w64(grow[0] || grow[1]) != 0) {
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const float alpha = grow[qt] ? __builtin_amdgcn_exp2f(mc_run[qt] - t2[qt]) : 1.f;
        l_run[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2 * NDT; ++dt)
#pragma unroll
          for (int r = 0; r < 4; ++r) o_acc[dt][qt][r] *= alpha;
        mc_run[qt] = grow[qt] ? t2[qt] : mc_run[qt];
      }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int kt = 2 * ks + (e >> 1), r = 2 * (e & 1);
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kt][qt][r], c, -mc_run[qt]));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kt][qt][r + 1], c, -mc_run[qt]));
          pq[ks][qt][e] = Elem<Tag>::pack2(p0, p1);
        }
  };

  // ---- schedule: identical to mha_pp_kernel (phases, barriers, waits)
  constexpr int LPT = 2 * L::LPW;                         // loads per wavefront per tile
#pragma unroll
  for (int t = 0; t < PA_AHEAD; ++t)
    if (t < nblk) issue_tile(t);
  if (nblk >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 15));
  else if (nblk == 2) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
  else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
  MLT_BARRIER();
  if (grp == 1) MLT_BARRIER();            // stagger: group 1 runs one phase behind

  // prologue: S_0 = K_0 Q^T, then the first two V_0 chunks
  {
    if (my_nblk > 0) {                                    // ka, va point into slot 0
#pragma unroll
      for (int i = 0; i < NDT; ++i) read_k_frag(0, i, fb[0][i]);
#pragma unroll
      for (int i = 0; i < NDT; ++i) read_k_frag(1, i, fb[1][i]);
      MLT_SB();
#pragma unroll
      for (int ch = 0; ch < 4; ++ch)
#pragma unroll
        for (int i = 0; i < NDT; ++i) {
          mfma_k(ch, i, fb[ch & 1][i]);
          MLT_SB();
          if (ch < 2) read_k_frag(ch + 2, i, fb[ch & 1][i]);
          else read_v_chunk_frag(ch - 2, i, fb[ch & 1][i]);
          MLT_SB();
        }
    }
    if (grp == 1) {
      if (nblk >= 3) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    }
    MLT_BARRIER();
  }

  int slot_off = 0;                                       // byte offset of tile j's slot
  for (int j = 0; j < nblk; ++j) {
    const int slot_off_next = slot_off + L::SLOT_B == L::SMEM ? 0 : slot_off + L::SLOT_B;
    const bool active = j < my_nblk;                       // wavefront-uniform
    const bool active_next = j + 1 < my_nblk;
    // ---- X_j
    if (j + PA_AHEAD < nblk) issue_tile(j + PA_AHEAD);
    __builtin_amdgcn_sched_barrier(0);
    if (active) {
      softmax_tile(j);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) asm volatile("" : "+v"(pq[ks][qt]));
    }
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 0) {
      const int newer = (j + 3 < nblk ? 1 : 0) + (j + 2 < nblk ? 1 : 0);
      if (newer == 2) __builtin_amdgcn_s_waitcnt(wait_imm(2 * LPT, 0));
      else if (newer == 1) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 0));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
    } else {
      __builtin_amdgcn_s_waitcnt(wait_imm(63, 0));
    }
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    if (D == 128) __builtin_amdgcn_s_setprio(1);
    // ---- C_j: O^T += V_j^T P_j^T (V chunks 0..3), then S_{j+1}^T = K_{j+1} Q^T (K chunks 0..3),
    // then the first two V_{j+1} chunks into the buffers; chunk n's MFMAs alternate with the reads
    // of chunk n+2. The fragment addresses move on to the slot of tile j+1 on the way.
    if (active) {
      const uint32_t dslot = (uint32_t)(slot_off_next - slot_off);
#pragma unroll
      for (int cg = 0; cg < 4; ++cg)
#pragma unroll
        for (int t = 0; t < NDT; ++t) {
          mfma_v(cg, t, fb[cg & 1][t]);
          MLT_SB();
          if (cg < 2) read_v_chunk_frag(cg + 2, t, fb[cg & 1][t]);
          else read_k_frag(cg - 2, t, fb[cg & 1][t]);
          if (cg == 0) ka[t] += dslot;
          if (cg == 3) va[t] += dslot;
          MLT_SB();
        }
      if (active_next) {
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
          for (int i = 0; i < NDT; ++i) {
            mfma_k(ch, i, fb[ch & 1][i]);
            MLT_SB();
            if (ch < 2) read_k_frag(ch + 2, i, fb[ch & 1][i]);
            else read_v_chunk_frag(ch - 2, i, fb[ch & 1][i]);
            MLT_SB();
          }
      }
      // row sums of the ROUNDED weights, behind the last MFMA (see mha_pp_kernel)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          l_run[0] = Elem<Tag>::add_pair(pq[ks][0][e], l_run[0]);
          l_run[1] = Elem<Tag>::add_pair(pq[ks][1][e], l_run[1]);
        }
      asm volatile("" : "+v"(l_run[0]), "+v"(l_run[1]));
    }
    if (D == 128) __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    if (grp == 1) {
      if (j + 3 < nblk) __builtin_amdgcn_s_waitcnt(wait_imm(LPT, 15));
      else __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    }
    MLT_BARRIER();
    __builtin_amdgcn_sched_barrier(0);
    slot_off = slot_off_next;
  }
#undef MLT_SB
  if (grp == 0) MLT_BARRIER();            // same barrier count for both groups

  // ---- epilogue: O = O^T / l, l summed over the four lane groups; 4 consecutive d per store
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const float inv = 1.f / four_groups_sum(l_run[qt]);
    if (my_q[qt] < Sq) {
      uint16_t* op = O + ((int64_t)bh * Sq + my_q[qt]) * D + 4 * g4;
#pragma unroll
      for (int dt = 0; dt < 2 * NDT; ++dt) {
        u32x2 w;
        w[0] = Elem<Tag>::pack2(o_acc[dt][qt][0] * inv, o_acc[dt][qt][1] * inv);
        w[1] = Elem<Tag>::pack2(o_acc[dt][qt][2] * inv, o_acc[dt][qt][3] * inv);
        *reinterpret_cast<u32x2_mem*>(op + dt * 16) = w;
      }
    }
  }
}

template <typename Tag, int D, bool CAUSAL, int MS>
int launch_mha_pp(const MhaArgs& a, hipStream_t s) {
  typedef PaCfg<D> L;
  auto kern = MS == 16 ? mha_pp16_kernel<Tag, D, CAUSAL> : mha_pp_kernel<Tag, D, CAUSAL>;
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
  const int nq = (int)((a.Sq + PA_BM - 1) / PA_BM);
  const int64_t total = a.B * a.H * nq;
  if (total > 0x7fffffff) return MLT_ERR_UNSUPPORTED;
  const float LOG2E = 1.4426950408889634f;
  // c > 0 always: a zero scale becomes a positive one too small to move any weight off 1, which
  // keeps (-inf) * c = -inf for masked scores instead of NaN
  float c = (a.scale < 0 ? -a.scale : a.scale) * LOG2E;
  if (c < 1e-30f) c = 1e-30f;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(PA_NT), L::SMEM, s, a.Q, a.K, a.V, a.O,
                     (int)a.Sq, (int)a.Sk, nq, (int)total, device_xcds(), c, a.scale < 0 ? 1 : 0);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

// The persistent kernel: one workgroup per CU, at most one per item.
template <typename Tag, int D>
int launch_mha_ps(const MhaArgs& a, hipStream_t s) {
  static_assert(D == 128, "see mha_ps_ok");
  typedef PaCfg<D> L;
  auto kern = mha_ps_kernel<Tag, D>;
  static thread_local int configured_dev = -1;          // opt in to > 64 KB LDS once per device
  static thread_local int ncu = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MLT_ERR_DEVICE;
  if (configured_dev != dev) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                            L::SMEM) != hipSuccess ||
        hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        ncu <= 0) {
      (void)hipGetLastError();
      return MLT_ERR_LAUNCH;
    }
    configured_dev = dev;
  }
  const int nq = (int)((a.Sq + PA_BM - 1) / PA_BM);
  const int64_t total = a.B * a.H * nq;
  int64_t slots = ncu;
  // Tuning/test override: a smaller number of workgroups makes every workgroup walk through many
  // items even on a small problem
  if (a.ps_grid >= 1 && a.ps_grid < slots) slots = a.ps_grid;
  const unsigned grid = (unsigned)(total < slots ? total : slots);
  const float LOG2E = 1.4426950408889634f;
  float c = (a.scale < 0 ? -a.scale : a.scale) * LOG2E;   // c > 0 always, as in launch_mha_pp
  if (c < 1e-30f) c = 1e-30f;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(PA_NT), L::SMEM, s, a.Q, a.K, a.V, a.O,
                     (int)a.Sq, (int)a.Sk, nq, (int)total, device_xcds(), c, a.scale < 0 ? 1 : 0);
  return hipGetLastError() == hipSuccess ? MLT_OK : MLT_ERR_LAUNCH;
}

template <typename Tag, int MS>
int run_mha_pp_t(const MhaArgs& a, hipStream_t s) {
  if (a.D == 128) return a.causal ? launch_mha_pp<Tag, 128, true, MS>(a, s) : launch_mha_pp<Tag, 128, false, MS>(a, s);
  if (a.D == 64) return a.causal ? launch_mha_pp<Tag, 64, true, MS>(a, s) : launch_mha_pp<Tag, 64, false, MS>(a, s);
  return MLT_ERR_UNSUPPORTED;
}

}  // namespace

// Sk * D * 2 must fit the 32-bit per-lane byte offsets of the direct loads.
bool mha_pp_ok(const MhaArgs& a) { return (a.D == 64 || a.D == 128) && a.Sk * a.D * 2 < ((int64_t)1 << 31); }

// The persistent kernel takes the unmasked case with at least two key tiles per item; the item
// and stream-tile counters are 32-bit.
// D = 128 only: at the 128 registers that D = 64 is compiled for (two workgroups per CU) the compiler
// spills a Q register while its inline-assembly load is still in flight, which the schedule's
// own wait cannot cover (and the persistent form measured 10 % slower than the per-item kernel
// there anyway).
bool mha_ps_ok(const MhaArgs& a) {
  if (a.D != 128) return false;
  if (!mha_pp_ok(a) || a.causal || a.Sk <= PA_BN || a.Sq < 1 || a.B * a.H < 1) return false;
  const int64_t nq = (a.Sq + PA_BM - 1) / PA_BM, nblk = (a.Sk + PA_BN - 1) / PA_BN;
  const int64_t total = a.B * a.H * nq;
  return total < ((int64_t)1 << 30) && total * nblk < ((int64_t)1 << 30);
}

int run_mha_ps(const MhaArgs& a, hipStream_t s) {
  if (!mha_ps_ok(a)) return MLT_ERR_UNSUPPORTED;
  return a.dtype == MLT_BF16 ? launch_mha_ps<bf16_tag, 128>(a, s) : launch_mha_ps<f16_tag, 128>(a, s);
}

int run_mha_pp(const MhaArgs& a, int mfma_size, hipStream_t s) {
  if (mfma_size == 16)
    return a.dtype == MLT_BF16 ? run_mha_pp_t<bf16_tag, 16>(a, s) : run_mha_pp_t<f16_tag, 16>(a, s);
  return a.dtype == MLT_BF16 ? run_mha_pp_t<bf16_tag, 32>(a, s) : run_mha_pp_t<f16_tag, 32>(a, s);
}

}  // namespace mlt
