#!/usr/bin/env python3
"""Times the library over sets of shapes and prints markdown tables (one MI355X, synthetic data).

  python3 paper_2503_14985_amd/sweep.py gemm [--torch] [--dtype fp16]
                                                          GEMM shapes: the square sweep, the LLM
                                                          shapes with B stored N x K, mid-size and
                                                          decode (skinny) shapes
  python3 paper_2503_14985_amd/sweep.py fa2              attention forward over the sweep of the
                                                          paper's FlashAttention-2 evaluation
                                                          (Section 4.2: 32k tokens in total,
                                                          hidden size 2048, with and without mask)

Each shape is launched back to back (best of two runs of n launches, HIP events on the launch
stream) with torch.randn inputs: N(0,1) for the square GEMMs and attention, N(0, 0.02^2) for
the shapes with B stored N x K. Times below about 12 us are bounded by the Python call, not by the
kernel; run the script under `rocprofv3 --kernel-trace --stats` for kernel-only durations.
--torch adds torch.matmul (hipBLASLt) on the same tensors as context.
"""
import argparse
import math
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GEMM_SHAPES = [
    # (M, N, K, B stored N x K)
    (1024, 1024, 1024, False), (2048, 2048, 2048, False), (3072, 3072, 3072, False),
    (4096, 4096, 4096, False), (8192, 8192, 8192, False), (8192, 8192, 8192, True),
    (4096, 14336, 4096, True), (4096, 4096, 14336, True), (8192, 28672, 8192, True),
    (1024, 4096, 4096, True), (512, 4096, 4096, True), (256, 4096, 4096, True), (128, 4096, 4096, True),
    (512, 8192, 8192, True), (256, 8192, 8192, True), (256, 14336, 4096, True), (512, 4096, 14336, True),
    (64, 4096, 4096, True), (64, 14336, 4096, True), (64, 28672, 8192, True), (64, 8192, 28672, True),
    (64, 131072, 4096, True), (32, 28672, 8192, True), (32, 8192, 28672, True),
    (16, 4096, 4096, True), (16, 28672, 8192, True), (16, 8192, 28672, True), (16, 131072, 4096, True),
    (1, 28672, 8192, True),
]


def _timeit(torch, fn, n):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def sweep_gemm(torch, binding, dev, with_torch, dt):
    head = "| M x N x K | B stored | kernel | us | TFLOP/s | GB/s (A+B+C once) |"
    print(head + (" torch us |" if with_torch else ""))
    print("|---|---|---|---|---|---|" + ("---|" if with_torch else ""))
    for (M, N, K, tb) in GEMM_SHAPES:
        std = 0.02 if tb else 1.0
        A = (torch.randn(M, K, device=dev, dtype=torch.float32) * std).to(dt)
        B = (torch.randn((N, K) if tb else (K, N), device=dev, dtype=torch.float32) * std).to(dt)
        C = torch.empty(M, N, device=dev, dtype=dt)
        n = 20 if M * N * K > 1e11 else 100
        ms = min(_timeit(torch, lambda: binding.mlt_gemm(A, B, C=C, transB=tb), n) for _ in range(2))
        line = "| %d x %d x %d | %s | `%s` | %.1f | %.0f | %.0f |" % (
            M, N, K, "N x K" if tb else "K x N", binding.mlt_last_kernel(), ms * 1e3,
            2.0 * M * N * K / ms / 1e9, 2.0 * (M * K + N * K + M * N) / ms / 1e6)
        if with_torch:
            tms = min(_timeit(torch, lambda: torch.matmul(A, B.t() if tb else B, out=C), n) for _ in range(2))
            line += " %.1f |" % (tms * 1e3)
        print(line, flush=True)


def sweep_fa2(torch, binding, dev):
    print("| heads x D | seq | batch | causal | dtype | kernel | ms | TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|")
    for (H, D) in [(32, 64), (16, 128)]:
        for S in [1024, 2048, 4096, 8192, 16384, 32768]:
            B = 32768 // S
            for causal in (False, True):
                for dt in (torch.float16, torch.bfloat16):
                    if dt == torch.bfloat16 and S not in (4096, 32768):
                        continue
                    q = torch.randn(B, H, S, D, device=dev, dtype=dt)
                    k, v = torch.randn_like(q), torch.randn_like(q)
                    o = torch.empty_like(q)
                    # causal: visible pairs only
                    flop = 4.0 * B * H * D * (S * (S + 1) / 2 if causal else S * S)
                    ms = min(_timeit(torch, lambda: binding.mlt_mha_fwd(q, k, v, 1 / math.sqrt(D), causal, O=o), 10)
                             for _ in range(2))
                    print("| %d x %d | %d | %d | %d | %s | `%s` | %.3f | %.0f |" % (
                        H, D, S, B, int(causal), "fp16" if dt == torch.float16 else "bf16",
                        binding.mlt_last_kernel(), ms, flop / ms / 1e9), flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["gemm", "fa2"])
    ap.add_argument("--torch", action="store_true", help="gemm: add torch.matmul on the same tensors")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default="bf16", help="gemm: element type")
    args = ap.parse_args()
    import torch
    from paper_2503_14985_amd import binding   # raises if libmlt.so is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    torch.manual_seed(0)
    if args.what == "gemm":
        sweep_gemm(torch, binding, dev, args.torch, torch.bfloat16 if args.dtype == "bf16" else torch.float16)
    else:
        sweep_fa2(torch, binding, dev)


if __name__ == "__main__":
    main()
