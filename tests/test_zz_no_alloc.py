"""The GEMM entry point that allocates nothing (mlt_gemm_noalloc): same result, bit for bit, as
mlt_gemm, with the partial products of a K split across workgroups in the library's fixed device
array instead of an allocated buffer. Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2503_14985_amd import inputs
import parity_util as pu

pytestmark = pytest.mark.gpu
BF16 = inputs.BF16


def _pair(M, N, K, seed, dev):
    A, B = inputs.gemm_inputs(M, N, K, BF16, seed, transB=True, std=0.02)
    return A, B, inputs.bits_to_torch(A, BF16, dev), inputs.bits_to_torch(B, BF16, dev)


def test_no_alloc_entry_point_matches_the_allocating_one():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    binding.mlt_diag_force_variant(gemm="auto")
    binding.mlt_diag_force_k_parts(0)
    try:
        # two calls in a row, the second on a smaller problem (its partial products cover only the
        # beginning of what the first call left in the scratch array); both split K by themselves
        for (M, N, K, seed) in ((64, 4096, 64 * 200, 70), (40, 1096, 64 * 130 + 8, 71)):
            A, B, tA, tB = _pair(M, N, K, seed, dev)
            want = binding.mlt_gemm(tA, tB, transB=True)
            name = binding.mlt_last_kernel()
            assert "splitk" in name, name
            got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
            binding.mlt_gemm_noalloc(tA, tB, got, transB=True)
            torch.cuda.synchronize()
            assert binding.mlt_last_kernel() == name
            assert torch.equal(got.view(torch.int16), want.view(torch.int16))
            pu.check_gemm(A, B, got, BF16, True, seed=seed)          # and both meet the oracle bound
        # a problem that needs no scratch at all goes through unchanged
        A, B, tA, tB = _pair(300, 520, 256, 72, dev)
        want = binding.mlt_gemm(tA, tB, transB=True)
        got = torch.empty_like(want)
        binding.mlt_gemm_noalloc(tA, tB, got, transB=True)
        torch.cuda.synchronize()
        assert "splitk" not in binding.mlt_last_kernel()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))
        # more scratch than the array holds (only a forced split asks for that): refused, C untouched
        binding.mlt_diag_force_k_parts(8)
        M, N, K = 1100, 1024, 64 * 80                                  # 8 * M * N * 4 bytes > 32 MiB
        tA = torch.zeros((M, K), dtype=torch.bfloat16, device=dev)
        tB = torch.zeros((N, K), dtype=torch.bfloat16, device=dev)
        got = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=dev)
        with pytest.raises(binding.MltError) as e:
            binding.mlt_gemm_noalloc(tA, tB, got, transB=True)
        assert e.value.status == binding.MLT_ERR_SCRATCH
        torch.cuda.synchronize()
        assert torch.all(got == 7.0)
    finally:
        binding.mlt_diag_force_k_parts(0)


def test_no_alloc_entry_point_inside_a_captured_graph():
    """What the entry point is for: a K-split GEMM captured into a HIP graph (on the capture stream
    the allocating entry point would have to hipMalloc its scratch in the middle of the capture).
    Replayed several times, with eager work in between and new input contents, against the eager
    result of mlt_gemm on the same contents."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    binding.mlt_diag_force_variant(gemm="auto")
    binding.mlt_diag_force_k_parts(0)
    M, N, K = 64, 2048, 64 * 160
    A, B, tA, tB = _pair(M, N, K, 80, dev)
    _, _, oA, oB = _pair(M, N, K, 81, dev)
    eager = binding.mlt_gemm(tA, tB, transB=True)
    assert "splitk" in binding.mlt_last_kernel()
    static = torch.empty_like(eager)
    binding.mlt_gemm_noalloc(tA, tB, static, transB=True)      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.mlt_gemm_noalloc(tA, tB, static, transB=True)
    for rep in range(4):
        if rep == 2:
            tA.copy_(oA)
            tB.copy_(oB)
            eager = binding.mlt_gemm(tA, tB, transB=True)
        static.fill_(0)
        graph.replay()
        other = binding.mlt_gemm(oA, oB, transB=True)           # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(static.view(torch.int16), eager.view(torch.int16)), "replay %d" % rep
        del other
