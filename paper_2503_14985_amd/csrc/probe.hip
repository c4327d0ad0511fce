// Diagnostic kernel behind mlt_probe_mfma: the rate at which the whole chip executes bf16
// 32x32x16 MFMAs when nothing else limits them. Every wavefront keeps 8 accumulator tiles and 24
// operand fragments in registers and issues MFMAs back to back, 8 wavefronts per workgroup, one
// workgroup per CU slot. The operand VALUES come from the caller: the rate depends on them,
// because the chip lowers its clock under the power that toggling operand bits costs (all-zero
// operands run at the nominal clock, N(0,1) operands do not). Benchmarks report this measured
// ceiling next to the nominal peak.
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {

namespace {

__global__ __launch_bounds__(512) void mfma_rate_kernel(int iters, const u32x4* __restrict__ data,
                                                        float* __restrict__ sink) {
  const int tid = threadIdx.x;
  bf16x8 a[4][4], b[4][2];
  const int base = tid & 511;                               // 16-byte words 0 .. 4095 are read
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[kk][i] = __builtin_bit_cast(bf16x8, data[base + (kk * 6 + i) * 128]);
#pragma unroll
    for (int j = 0; j < 2; ++j) b[kk][j] = __builtin_bit_cast(bf16x8, data[base + (kk * 6 + 4 + j) * 128 + 512]);
  }
  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(a[kk][i], b[kk][j], acc[i][j]);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  if (s == 12345.678f) sink[0] = s;                         // keeps the loop alive, practically never stores
}

}  // namespace

// 32 MFMAs of 32*32*16*2 flop per wavefront and iteration
double run_mfma_probe(int iters, int nblocks, const void* data, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(nblocks), dim3(512), 0, s, iters,
                     reinterpret_cast<const u32x4*>(data), sink);
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)nblocks * 8.0 * iters * 32.0 * 32768.0;
}

}  // namespace mlt
