"""Seeded random shapes through the library's own kernel choice, every output element checked
against the fp64 oracle: the shapes fall on both sides of every routing boundary (general / tile
kernels of four sizes with and without the K split / two-group kernel / skinny kernels, per-item
and persistent attention, masked and not) and have ragged ends almost always."""
import math
import os

import numpy as np
import pytest

from paper_2503_14985_amd import inputs
import parity_util as pu

pytestmark = pytest.mark.gpu
BF16, FP16 = inputs.BF16, inputs.FP16


@pytest.fixture(autouse=True)
def _announce(request):
    print("\n[case] %s" % request.node.name, flush=True)
    from paper_2503_14985_amd import binding
    binding.mlt_diag_force_variant(gemm="auto", mha="auto")
    binding.mlt_diag_set_persistent_grid(0)
    yield


def _gemm_case(rng, kind):
    if kind == "any":            # any alignment: mostly the general kernel
        M, N, K = (int(rng.integers(1, 400)) for _ in range(3))
    elif kind == "fast":         # 16-byte vector access: the tile kernels
        M = int(rng.integers(1, 900))
        N = 8 * int(rng.integers(1, 110))
        K = 8 * int(rng.integers(1, 150))
    elif kind == "k64":          # K a multiple of 64: the direct-to-LDS kernels are eligible
        M = int(rng.integers(200, 1400))
        N = 8 * int(rng.integers(100, 260))
        K = 64 * int(rng.integers(1, 12))
    else:                        # "skinny": short A against a wide B stored N x K
        M = int(rng.integers(1, 70))
        N = int(rng.integers(1024, 20000))
        K = 8 * int(rng.integers(1, 300))
    return M, N, K


@pytest.mark.parametrize("kind,count", [("any", 12), ("fast", 14), ("k64", 10), ("skinny", 12)])
def test_random_gemm_shapes(kind, count):
    from paper_2503_14985_amd import binding
    rng = np.random.default_rng({"any": 101, "fast": 102, "k64": 103, "skinny": 104}[kind])
    seen = set()
    for i in range(count):
        M, N, K = _gemm_case(rng, kind)
        transB = True if kind == "skinny" else bool(rng.integers(0, 2))
        dtype = BF16 if rng.integers(0, 2) else FP16
        A, B = inputs.gemm_inputs(M, N, K, dtype, 1000 + i, std=0.02 if kind == "skinny" else 1.0, transB=transB)
        C = pu.run_gemm(A, B, dtype, transB=transB)
        st = pu.check_gemm(A, B, C, dtype, transB, seed=i)
        name = binding.mlt_last_kernel()
        seen.add(name)
        print("   %4d x %5d x %5d transB=%d %s kernel=%s %s" % (M, N, K, transB, "bf16" if dtype == BF16 else "fp16", name, st), flush=True)
    print("   kernels seen:", sorted(seen), flush=True)
    assert len(seen) >= (1 if kind == "any" else 2)


@pytest.mark.parametrize("D", [64, 128])
def test_random_attention_shapes(D):
    from paper_2503_14985_amd import binding
    rng = np.random.default_rng(200 + D)
    seen = set()
    for i in range(14):
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        Sq, Sk = int(rng.integers(1, 800)), int(rng.integers(1, 800))
        causal = bool(rng.integers(0, 2))
        dtype = BF16 if rng.integers(0, 2) else FP16
        scale = float(rng.choice([1.0 / math.sqrt(D), 0.3 / math.sqrt(D), -1.0 / math.sqrt(D)]))
        Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, dtype, 2000 + i)
        O = pu.run_mha(Q, K, V, scale, causal, dtype)
        st = pu.check_mha(Q, K, V, O, scale, causal, dtype, seed=i)
        name = binding.mlt_last_kernel()
        seen.add(name)
        print("   B%d H%d Sq%d Sk%d causal=%d %s scale=%.3f kernel=%s %s" % (
            B, H, Sq, Sk, causal, "bf16" if dtype == BF16 else "fp16", scale, name, st), flush=True)
    print("   kernels seen:", sorted(seen), flush=True)
    assert len(seen) >= 2
