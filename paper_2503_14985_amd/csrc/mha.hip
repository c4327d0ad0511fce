// Attention forward: choice of the kernel for a problem (the kernels are in mha_pp.hip).
//
// All of them follow the FlashAttention-2 forward of the paper (arXiv 2503.14985, Section 2.5,
// Algorithm 1) with the row-only partition of its warpsPerCTA = [numWarps, 1]: workgroup =
// 8 wavefronts x 32 query rows of one (batch, head), key tile 64.
#include "mha_tile.h"
#include "mlt_internal.h"

namespace mlt {

MhaPlan plan_mha(const MhaArgs& a) {
  MhaPlan p;
  // Sk * D * 2 has to fit the 32-bit per-lane byte offsets of the direct global->LDS loads
  if ((a.D != 64 && a.D != 128) || !mha_pp_ok(a)) return p;
  p.supported = true;
  p.bm = PA_BM; p.bn = PA_BN; p.waves = PA_NT / 64;
  // Default: 32x32x16 MFMAs. Measured for D = 128: the 16x16x32 form is 3 % faster in back-to-back
  // launches but 2 % slower when it alternates with the GEMM; for D = 64 it does not fit the 128
  // registers that let two workgroups share a CU (-6 %).
  p.mfma_size = a.forced == MHA_PP16 ? 16 : 32;
  // The persistent form runs only on request. Measured, unmasked, 2048 items, time per item
  // against the per-item kernel: D = 128 gains 25 % at 2 key tiles per item, 8 % at 4, 3 % at 8
  // and loses 1.5 % at 16, 3 % at 32 and 4 % at 64 (its loop carries the item bookkeeping). It is
  // not the automatic choice even for short sequences: it fetches the next item's Q operand with
  // loads the compiler cannot see into registers the compiler manages, which holds for the
  // compiler this library is built with (the build's own check of the generated code and the
  // parity tests say so) but is not a property of the source. D = 64 has no persistent form
  // (mha_ps_ok). Where the forced form cannot run, the default kernel does.
  p.persistent = a.forced == MHA_PS && mha_ps_ok(a);
  if (p.persistent) {
    p.mfma_size = 32;
    p.name = "mha_fwd_d128_256x64_ps";
  } else if (p.mfma_size == 16) {
    if (a.D == 128) p.name = a.causal ? "mha_fwd_d128_causal_256x64_pp16" : "mha_fwd_d128_256x64_pp16";
    else p.name = a.causal ? "mha_fwd_d64_causal_256x64_pp16" : "mha_fwd_d64_256x64_pp16";
  } else {
    if (a.D == 128) p.name = a.causal ? "mha_fwd_d128_causal_256x64_pp" : "mha_fwd_d128_256x64_pp";
    else p.name = a.causal ? "mha_fwd_d64_causal_256x64_pp" : "mha_fwd_d64_256x64_pp";
  }
  return p;
}

int run_mha(const MhaArgs& a, const MhaPlan& p, hipStream_t s) {
  if (!p.supported) return MLT_ERR_UNSUPPORTED;
  if (p.persistent) return run_mha_ps(a, s);
  return run_mha_pp(a, p.mfma_size, s);
}

}  // namespace mlt
