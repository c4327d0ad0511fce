// Shared device-side vocabulary for the gfx950 kernels: 16-bit vector types, MFMA wrappers,
// LDS helpers. Wave64 only; every layout fact below was checked on hardware with one-hot probes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mlt.h"

namespace mlt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
// Every 16-byte memory access (global or LDS) goes through this one type, marked may_alias: the
// same LDS bytes are written as raw dwords and read back as 16-bit vectors, and type-based alias
// analysis would otherwise be free to treat those reads as unrelated to the writes.
typedef u32x4 __attribute__((may_alias)) u32x4_mem;
typedef u32x2 __attribute__((may_alias)) u32x2_mem;

#define MLT_LDS __attribute__((address_space(3)))

// Workgroup barrier of the pipelined kernels (the ones that order their direct-to-LDS loads with
// hand-counted s_waitcnt values). In the debug build (-DMLT_DEBUG_BARRIERS, libmlt_dbg.so) every
// such barrier first waits for ALL of the wavefront's outstanding memory operations and is taken
// twice, which changes the timing of every hand-off and makes any wait count that is too lax
// harmless there: since every result is a fixed function of the inputs (fixed summation orders),
// the two builds must agree bit for bit, and a tile read before it has landed, or a slot
// overwritten while still being read, shows as a difference between them.
#ifdef MLT_DEBUG_BARRIERS
#define MLT_BARRIER()                                                   \
  do {                                                                  \
    __builtin_amdgcn_s_waitcnt(0x0070); /* vmcnt(0) lgkmcnt(0) */       \
    __builtin_amdgcn_s_barrier();                                       \
    __builtin_amdgcn_s_barrier();                                       \
  } while (0)
#else
#define MLT_BARRIER() __builtin_amdgcn_s_barrier()
#endif

typedef __attribute__((address_space(3))) void* lptr_t;   // cast of a __shared__ pointer to its LDS byte address

// s_waitcnt immediate (gfx9 encoding: vmcnt [3:0]+[15:14], expcnt [6:4] left at its maximum,
// lgkmcnt [11:8]); vm = 63 / lgkm = 15 leave that counter alone
constexpr int wait_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | 0x70 | (lgkm << 8); }

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) straight into LDS at
// lds_addr + 16 * lane. Inline assembly on purpose: the compiler would order every later LDS read
// behind such a load (s_waitcnt vmcnt(0)), which would serialise the pipelines built on it; the
// kernels' own explicit waits and barriers establish the ordering instead.
__device__ __forceinline__ void load_lds16(const void* base, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(base)
               : "memory", "m0");
}

// Loads of data that is read exactly once (a streamed operand): the non-temporal form. Measured on
// a read-only sweep over 2 GiB: 7.1 TB/s against 6.3 TB/s for plain loads.
__device__ __forceinline__ u32x4 load_stream16(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
// the direct-to-LDS load in the same form
__device__ __forceinline__ void load_lds16_stream(const void* base, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
               :
               : "s"(lds_addr), "v"(voff), "s"(base)
               : "memory", "m0");
}

// Workgroup ids are dealt round-robin to the chip's XCDs (nxcd of them, from the device
// attributes), each with its own L2. This undoes the deal: XCD x owns one contiguous range of the
// `total` logical ids, so that workgroups that share operands can be made to share an L2.
__device__ __forceinline__ int logical_block(int bid, int total, int nxcd) {
  const int q = total / nxcd, rem = total % nxcd;
  const int xcd = bid % nxcd, idx = bid / nxcd;
  return xcd * q + (xcd < rem ? xcd : rem) + idx;
}

// Workgroup id -> C tile: logical ids walk the tiles in column-major order inside bands of GROUP_M
// tile rows, so that the workgroups resident on one XCD at a time share A row panels and B column
// panels.
template <int GROUP_M>
__device__ __forceinline__ void tile_of_block(int bid, int nbm, int nbn, int nxcd, int& tm, int& tn) {
  const int logical = logical_block(bid, nbm * nbn, nxcd);
  const int per_group = GROUP_M * nbn;
  const int g = logical / per_group;
  const int first_m = g * GROUP_M;
  const int rows = (nbm - first_m) < GROUP_M ? (nbm - first_m) : GROUP_M;
  const int in_g = logical % per_group;
  tm = first_m + in_g % rows;
  tn = in_g / rows;
}

struct bf16_tag {};
struct f16_tag {};

// Element traits: the 8-wide MFMA operand type and the fp32 -> 16-bit conversion (RNE).
template <typename Tag> struct Elem;
template <> struct Elem<bf16_tag> {
  typedef bf16x8 vec8;
  static __device__ __forceinline__ uint16_t from_f32(float x) {
    __bf16 h = (__bf16)x;  // v_cvt_pk_bf16_f32: round-to-nearest-even
    return __builtin_bit_cast(uint16_t, h);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
  }
  static __device__ __forceinline__ float to_f32(uint16_t bits) {
    return __builtin_bit_cast(float, (uint32_t)bits << 16);
  }
  // acc + lo + hi of a packed pair, exact in fp32 (v_dot2c_f32_bf16 against (1, 1))
  static __device__ __forceinline__ float add_pair(uint32_t packed, float acc) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), ones, acc, false);
  }
};
template <> struct Elem<f16_tag> {
  typedef f16x8 vec8;
  static __device__ __forceinline__ uint16_t from_f32(float x) {
    _Float16 h = (_Float16)x;  // v_cvt_f16_f32: round-to-nearest-even
    return __builtin_bit_cast(uint16_t, h);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 v = {lo, hi};
    f16x2 h = __builtin_convertvector(v, f16x2);
    return __builtin_bit_cast(uint32_t, h);
  }
  static __device__ __forceinline__ float to_f32(uint16_t bits) {
    return (float)__builtin_bit_cast(_Float16, bits);
  }
  // acc + lo + hi of a packed pair (v_dot2c_f32_f16 against (1, 1))
  static __device__ __forceinline__ float add_pair(uint32_t packed, float acc) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, packed), ones, acc, false);
  }
};

// One element of the GEMM result: rounded to the 16-bit type and stored (the default), or added
// to the fp32 value already there (the paper's C += A*B with an fp32 C, Section 2 / Listing 1;
// `idx` then counts fp32 elements).
template <typename Tag>
__device__ __forceinline__ void store_c(uint16_t* C, int64_t idx, float v, int acc32) {
  if (acc32) reinterpret_cast<float*>(C)[idx] += v;
  else C[idx] = Elem<Tag>::from_f32(v);
}

// Epilogue word of the GEMM kernels: bit 0 = add into an fp32 C (no bias, no activation);
// bit 3 = store the fp32 accumulator as it is (a partial product of a K split across workgroups:
// C then points at this part's slice of the fp32 scratch); otherwise bits 1..2 = activation
// applied to acc + bias[col] before rounding to the 16-bit C.
enum { EPI_ACC32 = 1, EPI_ACT_SHIFT = 1, EPI_ACT_MASK = 3, EPI_PART32 = 8, ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };
__device__ __forceinline__ float epi_act(float v, int act) {
  if (act == ACT_RELU) return v > 0.f ? v : 0.f;
  if (act == ACT_GELU) return 0.5f * v * (1.f + erff(v * 0.70710678118654752f));   // v * Phi(v)
  return v;
}
// The three ways a kernel's result elements leave: `each(fn)` calls fn(index into C, column, value)
// for every element this lane owns that lies inside the matrix.
template <typename Tag, typename Each>
__device__ __forceinline__ void gemm_epilogue(Each&& each, uint16_t* C, int epi, const uint16_t* bias) {
  if (epi & EPI_PART32) {
    each([&](int64_t idx, int, float v) { reinterpret_cast<float*>(C)[idx] = v; });
  } else if (epi & EPI_ACC32) {
    each([&](int64_t idx, int, float v) { reinterpret_cast<float*>(C)[idx] += v; });
  } else if (epi == 0 && bias == nullptr) {
    each([&](int64_t idx, int, float v) { C[idx] = Elem<Tag>::from_f32(v); });
  } else {
    const int act = (epi >> EPI_ACT_SHIFT) & EPI_ACT_MASK;
    each([&](int64_t idx, int col, float v) {
      if (bias) v += Elem<Tag>::to_f32(bias[col]);
      C[idx] = Elem<Tag>::from_f32(epi_act(v, act));
    });
  }
}

// D(32x32) += A(32x16) * B(16x32). Lane l supplies A[l%32][8*(l/32) .. +7] and
// B[8*(l/32) .. +7][l%32]; it owns D[8*(r/4) + 4*(l/32) + r%4][l%32] in register r (0..15).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
// D(16x16) += A(16x32) * B(32x16). Lane l supplies A[l%16][8*(l/16) .. +7] and
// B[8*(l/16) .. +7][l%16]; it owns D[4*(l/16) + r][l%16] in register r (0..3).
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// 16-byte LDS read of 8 consecutive 16-bit elements at a byte offset.
template <typename V8>
__device__ __forceinline__ V8 lds_read8(const char* smem, int byte_off) {
  const u32x4 raw = *reinterpret_cast<const u32x4_mem*>(smem + byte_off);
  return __builtin_bit_cast(V8, raw);
}

// Transposing LDS read (ds_read_b64_tr_b16). Within each group of 16 lanes, lane s = 4*j + c
// supplies the address of row j, columns 4c..4c+3 of a 4x16 block of 16-bit elements; lane i of
// the group receives column i of that block: (X[0][i], X[1][i], X[2][i], X[3][i]).
__device__ __forceinline__ s16x4 lds_read_tr4(const char* smem, int byte_off) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (MLT_LDS s16x4*)((MLT_LDS char*)smem + byte_off));
}

template <typename V8>
__device__ __forceinline__ V8 join_tr(s16x4 lo, s16x4 hi) {
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(V8, v);
}

}  // namespace mlt
