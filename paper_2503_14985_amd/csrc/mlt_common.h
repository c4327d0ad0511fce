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
