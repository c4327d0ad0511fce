"""Race check of the pipelined kernels: libmlt_dbg.so is the library compiled with
-DMLT_DEBUG_BARRIERS (every pipeline barrier first waits for all outstanding memory operations and
is taken twice). Every result of the library is a fixed function of its inputs, so the two builds
must agree bit for bit on every kernel family; a tile consumed before its load has landed, or a
ring slot refilled while a slower wavefront still reads it, would show as a difference."""
import ctypes
import math
import os

import pytest
import torch

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DBG = os.path.join(ROOT, "paper_2503_14985_amd", "libmlt_dbg.so")
_i64, _i32, _p, _f = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float


@pytest.fixture(scope="module")
def dbg():
    if not os.path.exists(DBG):
        pytest.skip("libmlt_dbg.so is not built (python -c 'import __graft_entry__ as g; g.build_debug_lib()')")
    lib = ctypes.CDLL(DBG)
    lib.mlt_gemm.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _p]
    lib.mlt_gemm_tiled.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _i32, _p]
    lib.mlt_mha_fwd.argtypes = [_i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _f, _i32, _i32, _p]
    lib.mlt_diag_force_variant.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    lib.mlt_last_kernel.restype = ctypes.c_char_p
    yield lib
    lib.mlt_diag_force_variant(b"auto", b"auto")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


GEMM_CASES = [
    # M, N, K, transB, forced variant, tiling hint (None: mlt_gemm)
    (1024, 768, 4096, False, "auto", None),       # two-group 256 x 256 kernel, row-major B
    (1000, 1000, 4096, True, "auto", None),       # the same, B stored N x K, ragged edge tiles
    (1000, 1000, 2048, False, "128pp16", None),   # the two-group kernel on 128 x 128 tiles, two workgroups per CU
    (1000, 1000, 2048, True, "128pp16", None),
    (1000, 1000, 2048, False, "128pp16k128", None),   # the same tile with K steps of 128
    (1000, 1000, 2048, True, "128pp16k128", None),
    (1024, 1024, 1024, False, "auto", 3),         # square hint: the 4-wavefront pipelined kernel
    (1024, 1024, 1024, True, "auto", 3),
    (300, 520, 1000, False, "auto", None),        # register-staged tile kernels
    (64, 4096, 64 * 200, True, "auto", None),     # K split across workgroups
    (16, 8192, 4096, True, "auto", None),         # streaming skinny kernel (LDS ring)
    (16, 4096, 4096, True, "auto", None),         # skinny kernel, K split inside the workgroup
    (32, 8192, 4096, True, "skinnydma", None),
]


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
def test_gemm_kernels_agree_with_the_debug_build(dbg, dt):
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    code = 0 if dt == torch.bfloat16 else 1
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    try:
        for (M, N, K, tb, variant, tiling) in GEMM_CASES:
            print("\n[case] %s" % ((M, N, K, tb, variant, tiling),), flush=True)
            A = torch.randn((M, K), generator=g, device=dev, dtype=torch.float32).to(dt)
            B = torch.randn((N, K) if tb else (K, N), generator=g, device=dev, dtype=torch.float32).to(dt)
            binding.mlt_diag_force_variant(gemm=variant)
            dbg.mlt_diag_force_variant(variant.encode(), None)
            if tiling is None:
                want = binding.mlt_gemm(A, B, transB=tb)
            else:
                want = binding.mlt_gemm_tiled(A, B, tiling, transB=tb)
            name = binding.mlt_last_kernel()
            got = torch.full_like(want, float("nan"))
            for _ in range(3):                     # a race need not strike on the first launch
                if tiling is None:
                    rc = dbg.mlt_gemm(M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), int(tb),
                                      got.data_ptr(), got.stride(0), code, _stream())
                else:
                    rc = dbg.mlt_gemm_tiled(M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), int(tb),
                                            got.data_ptr(), got.stride(0), code, tiling, _stream())
                assert rc == 0
                torch.cuda.synchronize()
                assert dbg.mlt_last_kernel().decode() == name
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), name
                want = binding.mlt_gemm(A, B, transB=tb) if tiling is None else binding.mlt_gemm_tiled(A, B, tiling, transB=tb)
    finally:
        binding.mlt_diag_force_variant(gemm="auto")


@pytest.mark.parametrize("variant", ["pp32", "pp16", "ps"])
@pytest.mark.parametrize("D", [64, 128])
def test_attention_kernels_agree_with_the_debug_build(dbg, variant, D):
    from paper_2503_14985_amd import binding
    if variant == "ps" and D == 64:
        pytest.skip("the persistent kernel has no D = 64 form")
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(6)
    try:
        binding.mlt_diag_force_variant(mha=variant)
        dbg.mlt_diag_force_variant(None, variant.encode())
        for (B, H, Sq, Sk, causal, dt) in ((2, 3, 1000, 1000, False, torch.bfloat16),
                                           (2, 3, 1000, 1000, True, torch.float16),
                                           (1, 2, 2048, 2048, False, torch.float16),
                                           (1, 2, 300, 2500, True, torch.bfloat16),
                                           (3, 40, 512, 512, False, torch.bfloat16)):
            if variant == "ps" and causal:
                continue
            print("\n[case] %s" % ((B, H, Sq, Sk, D, causal, dt),), flush=True)
            q = torch.randn((B, H, Sq, D), generator=g, device=dev, dtype=dt)
            k = torch.randn((B, H, Sk, D), generator=g, device=dev, dtype=dt)
            v = torch.randn((B, H, Sk, D), generator=g, device=dev, dtype=dt)
            scale = 1.0 / math.sqrt(D)
            want = binding.mlt_mha_fwd(q, k, v, scale, causal=causal)
            name = binding.mlt_last_kernel()
            got = torch.full_like(want, float("nan"))
            for _ in range(3):
                rc = dbg.mlt_mha_fwd(B, H, Sq, Sk, D, q.data_ptr(), k.data_ptr(), v.data_ptr(), got.data_ptr(),
                                     scale, int(causal), 0 if dt == torch.bfloat16 else 1, _stream())
                assert rc == 0
                torch.cuda.synchronize()
                assert dbg.mlt_last_kernel().decode() == name
                assert torch.equal(got.view(torch.int16), want.view(torch.int16)), name
                want = binding.mlt_mha_fwd(q, k, v, scale, causal=causal)
    finally:
        binding.mlt_diag_force_variant(mha="auto")
