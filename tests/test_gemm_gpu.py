"""GPU parity of mlt_gemm against the fp64 oracle (through the C ABI via the ctypes binding)."""
import os

import numpy as np
import pytest
import torch

from paper_2503_14985_amd import inputs
import parity_util as pu

pytestmark = pytest.mark.gpu
BF16, FP16 = inputs.BF16, inputs.FP16


@pytest.fixture(autouse=True)
def _announce(request):
    from paper_2503_14985_amd import binding
    print("\n[case] %s" % request.node.name, flush=True)
    binding.mlt_diag_force_variant(gemm="auto")
    binding.mlt_diag_force_k_parts(0)
    yield
    binding.mlt_diag_force_variant(gemm="auto")
    binding.mlt_diag_force_k_parts(0)


def _go(M, N, K, dtype, transB, dist="normal", std=1.0, seed=0, variant=None, **pads):
    from paper_2503_14985_amd import binding
    A, B = inputs.gemm_inputs(M, N, K, dtype, seed, dist=dist, std=std, transB=transB)
    binding.mlt_diag_force_variant(gemm=variant or "auto")
    C = pu.run_gemm(A, B, dtype, transB=transB, lda=pads.get("lda"), ldb=pads.get("ldb"),
                    ldc_pad=pads.get("ldc_pad", 0))
    st = pu.check_gemm(A, B, C, dtype, transB, seed=seed)
    print("   kernel=%s %s" % (binding.mlt_last_kernel(), st), flush=True)
    return binding.mlt_last_kernel(), st


def test_config1_bf16_512_uniform():
    name, _ = _go(512, 512, 512, BF16, False, dist="uniform")
    assert name.startswith("gemm_nn")


@pytest.mark.parametrize("variant", ["256", "256w8", "128w8", "64x128", "64", "128k2", "64x128k2", "64k4", "general"])
@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_small_multi_tile_ragged(variant, transB, dtype):
    # several tiles of every variant in both directions plus ragged tails in M, N and K
    _go(520, 776, 328, dtype, transB, variant=variant, seed=1)


@pytest.mark.parametrize("variant", ["256", "256w8", "128w8"])
@pytest.mark.parametrize("transB", [False, True])
def test_exact_tiles(variant, transB):
    _go(512, 768, 256, BF16, transB, variant=variant, seed=2)


@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(520, 776, 320), (512, 768, 256), (100, 40, 64), (257, 264, 128)])
def test_two_group_kernel(shape, transB, dtype):
    # the direct-to-LDS two-group kernel (16x16x32 MFMAs) on both of its tile sizes: K a multiple
    # of 64, ragged and exact M/N, one and many K steps
    M, N, K = shape
    name, _ = _go(M, N, K, dtype, transB, variant="256pp16", seed=6)
    assert name.endswith("256x256x64_w2x4_pp16")
    name, _ = _go(M, N, K, dtype, transB, variant="128pp16", seed=6)
    assert name.endswith("128x128x64_w2x4_pp16")


@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(520, 776, 384), (512, 768, 128), (100, 40, 256), (257, 264, 1280), (300, 263, 640)])
def test_two_group_kernel_k_steps_of_128(shape, transB, dtype):
    # the 128 x 128 tile with K steps of 128: one, few and many steps, ragged M / N, odd N with B
    # stored N x K; a K that is a multiple of 64 only falls back to the 64-deep form
    M, N, K = shape
    if not transB and N % 8:
        N += 8 - N % 8
    name, _ = _go(M, N, K, dtype, transB, variant="128pp16k128", seed=16)
    assert name.endswith("128x128x128_w2x4_pp16")
    name, _ = _go(M, N, K + 64, dtype, transB, variant="128pp16k128", seed=16)
    assert name.endswith("128x128x64_w2x4_pp16")


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("case", [(300, 263, 128, 0), (259, 520, 192, 1), (259, 520, 192, 3), (513, 262, 64, 2)])
def test_two_group_kernel_store_forms(case, dtype):
    # the 16x16x32 form stores pairs of columns as 32-bit words when N and ldc are even and falls
    # back to element stores otherwise: odd N (B stored N x K), odd and even padded ldc, odd M
    M, N, K, ldc_pad = case
    for variant in ("256pp16", "128pp16"):
        name, _ = _go(M, N, K, dtype, True, variant=variant, seed=13, ldc_pad=ldc_pad)
        assert name.endswith("_pp16")


@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(520, 776, 320), (512, 768, 256), (100, 40, 64), (257, 264, 128),
                                   (300, 520, 64 * 7)])
def test_four_wavefront_pipelined_kernel(shape, transB, dtype):
    # 2 x 2 wavefronts of 128 x 128 with the hand-pipelined K loop: one, two, three and more K steps
    # (the loop issues loads and prefetches past the last step into dead slots), ragged M/N
    M, N, K = shape
    name, _ = _go(M, N, K, dtype, transB, variant="256w4", seed=12)
    assert name.endswith("_swp")


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(16, 1024, 4096), (1, 1040, 512), (7, 1500, 264), (33, 2048, 8200),
                                   (64, 1024, 1000), (48, 1031, 4096 + 32),
                                   (16, 16400, 520), (40, 32 * 1024 + 8, 264)])   # 32 / 64 columns per workgroup
def test_skinny_kernel(shape, dtype):
    # M <= 64 with B stored N x K: one to four 16-row tiles, ragged N, K with and without a partial
    # last batch (K % 4096 != 0) and a partial last chunk (K % 32 != 0)
    M, N, K = shape
    name, _ = _go(M, N, K, dtype, True, std=0.02, seed=7, variant="skinny")
    assert "skinny" in name
    # the same problem through the tile kernel must agree with the oracle too (and is what a
    # row-major B or a larger M gets)
    name, _ = _go(M, N, K, dtype, True, std=0.02, seed=7, variant="128w8")
    assert "skinny" not in name


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(16, 1024, 512), (1, 1031, 520), (17, 2048, 4096 + 8), (64, 1040, 1024),
                                   (33, 4096, 8), (48, 1500, 7000), (16, 16 * 300 + 5, 1536),
                                   (20, 64 * 300 + 21, 1160), (16, 40965, 520), (8, 36880, 1536)])
def test_skinny_streaming_kernel(shape, dtype, form="skinnydma"):
    # B streamed through the LDS ring by persistent workgroups (stages of 16 columns x 512 k): one
    # to four 16-row tiles of A, ragged N (clamped rows), K below /
    # equal to / not a multiple of the stage, a single 8-wide K, and more column blocks than CUs
    # (several blocks per workgroup, the ring wrapping across block ends; the last two shapes give
    # a workgroup more blocks than one group holds: full and partial groups, odd and even numbers
    # of k stages)
    M, N, K = shape
    name, _ = _go(M, N, K, dtype, True, std=0.02, seed=8, variant=form)
    assert name.endswith("cols_stream")


@pytest.mark.parametrize("parts", [2, 4, 8])
@pytest.mark.parametrize("variant", ["64k4", "64x128k2", "128k2", "128w8", "64"])
@pytest.mark.parametrize("transB", [False, True])
def test_k_split_across_workgroups(variant, transB, parts):
    """The K steps of a tile split over 2, 4 or 8 workgroups (Section 4.1's memory-bound shapes: few
    tiles against a long K): fp32 partial tiles through the scratch, added in a fixed order by the
    second kernel, which also applies the epilogue. Ragged M and N, K not a multiple of the step
    (the last part is shorter, its last step partial), parts that do not divide the steps."""
    from paper_2503_14985_amd import binding
    binding.mlt_diag_force_k_parts(parts)
    for dtype, (M, N, K) in ((BF16, (200, 328, 64 * 67 + 8)), (FP16, (70, 136, 64 * 70))):
        name, _ = _go(M, N, K, dtype, transB, variant=variant, seed=50 + parts)
        assert name.endswith("_splitk%d" % parts), name
    # too few K steps for that many parts: the split is dropped, not the kernel
    name, _ = _go(100, 72, 64 * 4, BF16, transB, variant=variant, seed=51)
    assert "splitk" not in name


def test_k_split_results_do_not_depend_on_the_run():
    """Fixed-order reduction: the same call twice gives the same bits (no atomics), and the split
    result meets the oracle bound like the unsplit one."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    A, B = inputs.gemm_inputs(64, 1024, 64 * 96, BF16, 60, transB=True, std=0.02)
    tA, tB = inputs.bits_to_torch(A, BF16, dev), inputs.bits_to_torch(B, BF16, dev)
    binding.mlt_diag_force_k_parts(4)
    c1 = binding.mlt_gemm(tA, tB, transB=True).clone()
    c2 = binding.mlt_gemm(tA, tB, transB=True)
    torch.cuda.synchronize()
    assert "splitk4" in binding.mlt_last_kernel()
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))
    pu.check_gemm(A, B, c2, BF16, True, seed=60)


@pytest.mark.parametrize("parts", [2, 8])
def test_k_split_with_fp32_accumulate_and_fused_epilogue(parts):
    """The split's second kernel carries the epilogue: C(fp32) += A*B and act(A*B + bias)."""
    import oracle
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    binding.mlt_diag_force_k_parts(parts)
    binding.mlt_diag_force_variant(gemm="64k4")
    M, N, K = 130, 200, 64 * 70
    A, B = inputs.gemm_inputs(M, N, K, BF16, 61, transB=True)
    C0 = np.random.default_rng(61).standard_normal((M, N)).astype(np.float32) * 10.0
    Ct = torch.from_numpy(C0.copy()).to(dev)
    binding.mlt_gemm_acc(inputs.bits_to_torch(A, BF16, dev), inputs.bits_to_torch(B, BF16, dev), Ct, transB=True)
    torch.cuda.synchronize()
    assert binding.mlt_last_kernel().endswith("_splitk%d" % parts)
    Cref, T = oracle.gemm(A, B, BF16, transB=True)
    err = np.abs(Ct.double().cpu().numpy() - (C0.astype(np.float64) + Cref))
    bound = (K * 2.0 ** -24) * T + 2.0 ** -22 * (np.abs(C0) + T) + 1e-6
    assert np.all(err <= bound), "worst err/bound %.3f" % float(np.max(err / bound))
    bias = inputs.bias_input(N, BF16, 61, std=4.0)
    st = pu.run_check_gemm_bias_act(A, B, bias, 2, BF16, transB=True)
    assert binding.mlt_last_kernel().endswith("_splitk%d" % parts)
    print("   %s" % st, flush=True)


@pytest.mark.parametrize("shape", [(64, 8192, 28672), (512, 4096, 14336), (48, 8192, 28672 + 8)])
def test_k_split_is_chosen_for_few_tiles_against_a_long_k(shape):
    """Full-size memory-bound shapes in the launch configuration the library picks by itself."""
    M, N, K = shape
    name, _ = _go(M, N, K, BF16, True, std=0.02, seed=0)
    assert "splitk" in name, name


def test_skinny_routing():
    # one 16-row tile of A and B of 2^25 elements: the streaming kernel without any override
    name, _ = _go(16, 8192, 4096, BF16, True, std=0.02, seed=9)
    assert name.endswith("16cols_stream")
    name, _ = _go(16, 4096, 4096, BF16, True, std=0.02, seed=9)       # smaller B: K split over the wavefronts
    assert name.endswith("skinny_16cols_ksplit8")
    name, _ = _go(30, 4096, 2048, BF16, True, std=0.02, seed=9)
    assert name.endswith("skinny_16cols_ksplit8")
    # two row tiles against a large B: whichever of the streaming kernel and the tile kernels the
    # estimate favours (a long K with few columns goes to the tile kernels with K split across
    # workgroups, many columns stay with the streaming kernel or unsplit tiles)
    name, _ = _go(17, 8192, 4096, BF16, True, std=0.02, seed=9)
    assert "16cols_stream" in name or "_k" in name
    name, _ = _go(32, 4096, 28672, BF16, True, std=0.02, seed=9)
    assert "splitk" in name
    # taller A: the tile kernels (small tiles, K split inside the workgroup)
    name, _ = _go(40, 16384, 2048, FP16, True, std=0.02, seed=9)
    assert "skinny" not in name and "_k" in name
    name, _ = _go(64, 4096, 4096, BF16, True, std=0.02, seed=9)
    assert "64x64x64_w2x2_k4" in name


@pytest.mark.parametrize("variant", ["128k2", "64x128k2", "64k4"])
@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("K", [8, 64, 72, 128, 200, 64 * 5, 64 * 9 + 24, 2048])
def test_k_split_inside_the_workgroup(variant, transB, K):
    """The small-tile kernels with 2 to 4 groups of wavefronts per workgroup, each group on its own
    share of the K steps, summed through LDS: fewer K steps than groups (idle groups), uneven
    shares, a partial last step, many steps; ragged M and N."""
    for dtype in (BF16, FP16):
        name, _ = _go(200, 328, K, dtype, transB, variant=variant, seed=40 + K % 7)
        assert "_k" in name


@pytest.mark.parametrize("shape,tile", [((1024, 1024, 1024), "64x64x64_w2x2_k4"), ((2048, 2048, 2048), "128x128x128_w2x4_pp16"),
                                        ((3072, 3072, 3072), "256x256x64_w2x4_pp16"),
                                        ((512, 8192, 1024), "128x128x64_w2x4_k2"), ((512, 4096, 1024), "64x128x64_w2x4_k2"),
                                        ((256, 4096, 2048), "64x64x64_w2x2_k4"), ((2048, 2048, 2048 + 8), "128x128x64_w2x4_k2"),
                                        ((4096, 4096, 512), "256x256x64_w2x4_pp16"), ((1024, 1024, 256), "64x64x64_w2x2"),
                                        ((2048, 2048, 448), "128x128x64_w2x4")])
def test_tile_size_routing(shape, tile):
    """The workgroup tile is the one with the least estimated time over the whole grid: the
    256 x 256 two-group kernel once its tiles cover enough of the chip, 128 x 128 (two-group with
    K steps of 128 when one tile per CU runs long enough, register-staged otherwise), 64 x 128 or
    64 x 64 below that; sampled parity at the real size either way."""
    M, N, K = shape
    name, _ = _go(M, N, K, BF16, False, seed=21)
    assert name.endswith(tile), name


@pytest.mark.parametrize("shape", [(1, 1, 1), (37, 53, 29), (65, 63, 33), (16, 8, 8), (8, 16, 24),
                                   (255, 257, 64), (3, 1000, 2048)])
@pytest.mark.parametrize("transB", [False, True])
def test_odd_shapes(shape, transB):
    M, N, K = shape
    _go(M, N, K, BF16, transB, seed=3)
    _go(M, N, K, FP16, transB, seed=3)


@pytest.mark.parametrize("transB", [False, True])
def test_padded_leading_dimensions(transB):
    K, N = 200, 264
    _go(300, N, K, BF16, transB, seed=4, lda=K + 8, ldb=(K if transB else N) + 16, ldc_pad=5)
    # an even ldc keeps the paired 32-bit stores of the tile kernels: odd M, padding must stay untouched
    for variant in ("128w8", "64k4", "256"):
        _go(301, N, K, FP16, transB, seed=4, lda=K + 8, ldb=(K if transB else N) + 16, ldc_pad=6, variant=variant)
    from paper_2503_14985_amd import binding
    binding.mlt_diag_force_variant(gemm="auto")
    # unaligned leading dimensions must fall back to the general kernel and still be right
    name, _ = _go(70, N, K, BF16, transB, seed=4, lda=K + 3, ldb=(K if transB else N) + 1, ldc_pad=1)
    assert "general" in name


@pytest.mark.parametrize("variant,shape,transB", [("256pp16", (300, 264, 192), False), ("256pp16", (300, 264, 192), True),
                                                  ("128pp16", (300, 264, 192), False), ("128pp16", (300, 264, 192), True),
                                                  ("128pp16k128", (300, 264, 256), False), ("128pp16k128", (300, 264, 256), True),
                                                  ("256w4", (300, 264, 192), False),
                                                  ("256w4", (300, 264, 192), True), ("skinnydma", (16, 1100, 1032), True),
                                                  ("skinnydma", (40, 1100, 1032), True), ("skinny", (16, 1100, 1032), True)])
def test_padded_leading_dimensions_direct_load_kernels(variant, shape, transB):
    # row strides larger than the rows (NaN-filled padding that must never be read into a result
    # or written) through the kernels that address global memory with per-lane byte offsets
    M, N, K = shape
    name, _ = _go(M, N, K, BF16, transB, seed=14, variant=variant, std=0.05,
                  lda=K + 8, ldb=(K if transB else N) + 16, ldc_pad=5)
    assert "general" not in name
    name2, _ = _go(M, N, K, FP16, transB, seed=14, variant=variant, std=0.05,
                   lda=K + 24, ldb=(K if transB else N) + 8, ldc_pad=3)
    assert name2 == name


def test_k_zero_and_empty():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    A = torch.empty((5, 0), dtype=torch.bfloat16, device=dev)
    B = torch.empty((0, 7), dtype=torch.bfloat16, device=dev)
    C = torch.full((5, 7), float("nan"), dtype=torch.bfloat16, device=dev)
    binding.mlt_gemm(A, B, C=C)
    torch.cuda.synchronize()
    assert torch.all(C == 0)
    C0 = binding.mlt_gemm(torch.empty((0, 8), dtype=torch.float16, device=dev),
                          torch.empty((8, 4), dtype=torch.float16, device=dev))
    assert C0.shape == (0, 4)


def test_integer_exact_and_identity():
    """Small integers: fp32 accumulation is exact, so the GPU must equal the oracle exactly."""
    from paper_2503_14985_amd import binding
    rng = np.random.default_rng(5)
    M, N, K = 300, 264, 136
    a = rng.integers(-4, 5, (M, K)).astype(np.float32)
    b = rng.integers(-4, 5, (K, N)).astype(np.float32)
    A, B = inputs.to_bits(a, BF16), inputs.to_bits(b, BF16)
    C = pu.run_gemm(A, B, BF16)
    import oracle
    Cref, _ = oracle.gemm(A, B, BF16)
    # |C| <= 16*136 = 2176 needs 12 bits: not exact in bf16; compare after rounding the oracle
    want = np.array([oracle.round_to_dtype(v, BF16) for v in Cref.ravel()]).reshape(M, N)
    assert np.array_equal(C.double().cpu().numpy(), want)
    eye = inputs.to_bits(np.eye(256, dtype=np.float32), BF16)
    X = inputs.to_bits(rng.standard_normal((256, 256)).astype(np.float32), BF16)
    Y = pu.run_gemm(X, eye, BF16)
    assert np.array_equal(inputs.torch_to_bits(Y), X)
    Y = pu.run_gemm(eye, X, BF16, transB=True)             # I * (X^T stored as X) = X^T
    assert np.array_equal(inputs.torch_to_bits(Y), np.ascontiguousarray(X.T))


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("n", [1024, 2048, 4096, 8192])
def test_config2_square_sweep(dtype, n):
    _go(n, n, n, dtype, False, seed=0)


@pytest.mark.parametrize("shape", [(4096, 14336, 4096), (4096, 4096, 14336), (8192, 28672, 8192),
                                   (16, 4096, 4096)])
def test_config3_llm_shapes_transB(shape):
    M, N, K = shape
    _go(M, N, K, BF16, True, std=0.02, seed=0)


@pytest.mark.parametrize("shape,suffix", [((16, 28672, 8192), "16cols_stream"), ((1, 28672, 8192), "16cols_stream"),
                                          ((64, 28672, 4096), "_k"), ((16, 131072, 4096), "16cols_stream"),
                                          ((32, 8192, 28672), "_splitk4"), ((64, 8192, 28672), "_splitk4")])
def test_decode_shapes_streaming_kernels_full_size(shape, suffix):
    # the memory-bound decode GEMMs at their real sizes, in the launch configuration the library
    # picks (persistent workgroups, several column blocks each); sampled against the oracle
    M, N, K = shape
    name, _ = _go(M, N, K, BF16, True, std=0.02, seed=0)
    assert suffix in name


@pytest.mark.parametrize("variant", [None, "256pp16", "128pp16", "128w8", "general"])
@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_accumulate_into_fp32_c(variant, transB, dtype):
    """The paper's form of the GEMM (Listing 1): C(fp32) += A*B. Expected value: the fp32 C widened
    to double plus the oracle's fp64 product; error budget: fp32 accumulation over K terms plus the
    final fp32 addition (no 16-bit rounding anywhere)."""
    import oracle
    from paper_2503_14985_amd import binding
    M, N, K = 520, 776, 320
    A, B = inputs.gemm_inputs(M, N, K, dtype, 8, transB=transB)
    rng = np.random.default_rng(8)
    C0 = rng.standard_normal((M, N)).astype(np.float32) * 10.0
    dev = torch.device("cuda:0")
    Ct = torch.from_numpy(C0.copy()).to(dev)
    binding.mlt_diag_force_variant(gemm=variant or "auto")
    At, Bt = inputs.bits_to_torch(A, dtype, dev), inputs.bits_to_torch(B, dtype, dev)
    binding.mlt_gemm_acc(At, Bt, Ct, transB=transB)
    binding.mlt_gemm_acc(At, Bt, Ct, transB=transB)          # twice: C0 + 2 A*B
    torch.cuda.synchronize()
    print("   kernel=%s" % binding.mlt_last_kernel(), flush=True)
    Cref, T = oracle.gemm(A, B, dtype, transB=transB)
    want = C0.astype(np.float64) + 2.0 * Cref
    err = np.abs(Ct.double().cpu().numpy() - want)
    bound = 2.0 * (K * 2.0 ** -24) * T + 2.0 ** -22 * (np.abs(C0) + 2.0 * T) + 1e-6
    assert np.all(err <= bound), "worst err/bound %.3f" % float(np.max(err / bound))


@pytest.mark.parametrize("transB", [False, True])
def test_k_steps_of_128_fp32_accumulate_and_fused_epilogue(transB):
    """The 128 x 128 two-group kernel with K steps of 128 through the other two epilogues: fp32
    C += A*B (twice) and act(A*B + bias)."""
    import oracle
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    M, N, K = 392, 520, 384
    try:
        binding.mlt_diag_force_variant(gemm="128pp16k128")
        for dtype in (BF16, FP16):
            A, B = inputs.gemm_inputs(M, N, K, dtype, 31, transB=transB)
            At, Bt = inputs.bits_to_torch(A, dtype, dev), inputs.bits_to_torch(B, dtype, dev)
            C0 = np.random.default_rng(32).standard_normal((M, N)).astype(np.float32)
            Ct = torch.from_numpy(C0.copy()).to(dev)
            binding.mlt_gemm_acc(At, Bt, Ct, transB=transB)
            binding.mlt_gemm_acc(At, Bt, Ct, transB=transB)
            torch.cuda.synchronize()
            assert binding.mlt_last_kernel().endswith("128x128x128_w2x4_pp16")
            Cref, T = oracle.gemm(A, B, dtype, transB=transB)
            err = np.abs(Ct.double().cpu().numpy() - (C0.astype(np.float64) + 2.0 * Cref))
            bound = 2.0 * (K * 2.0 ** -24) * T + 2.0 ** -22 * (np.abs(C0) + 2.0 * T) + 1e-6
            assert np.all(err <= bound), "worst err/bound %.3f" % float(np.max(err / bound))
            for act in (0, 1, 2):
                bias = inputs.bias_input(N, dtype, 33, std=4.0)
                pu.run_check_gemm_bias_act(A, B, bias, act, dtype, transB=transB)
                assert binding.mlt_last_kernel().endswith("128x128x128_w2x4_pp16")
    finally:
        binding.mlt_diag_force_variant(gemm="auto")


def test_accumulate_edge_cases():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    C = torch.full((5, 7), 3.25, dtype=torch.float32, device=dev)
    binding.mlt_gemm_acc(torch.empty((5, 0), dtype=torch.bfloat16, device=dev),
                         torch.empty((0, 7), dtype=torch.bfloat16, device=dev), C)
    torch.cuda.synchronize()
    assert torch.all(C == 3.25)                                # K = 0: C += 0
    # a skinny shape must not take the 16-bit-output skinny kernel
    A = torch.ones((4, 64), dtype=torch.bfloat16, device=dev)
    B = torch.ones((2048, 64), dtype=torch.bfloat16, device=dev)
    C = torch.zeros((4, 2048), dtype=torch.float32, device=dev)
    binding.mlt_gemm_acc(A, B, C, transB=True)
    torch.cuda.synchronize()
    assert "skinny" not in binding.mlt_last_kernel() and torch.all(C == 64.0)
    with pytest.raises(ValueError):
        binding.mlt_gemm_acc(A, B, torch.zeros((4, 2048), dtype=torch.bfloat16, device=dev), transB=True)


@pytest.mark.parametrize("act", [0, 1, 2])
@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("variant,shape", [("256pp16", (520, 776, 320)), ("128pp16", (520, 776, 320)), ("256", (300, 264, 200)),
                                           ("128w8", (260, 392, 136)), ("general", (70, 53, 29)),
                                           (None, (16, 2048, 512))])
def test_fused_bias_activation(variant, shape, with_bias, act):
    """C = act(A*B + bias) through every kernel family's epilogue (several tiles, ragged edges);
    the last shape would take the skinny kernel, which has no fused epilogue, and must not."""
    from paper_2503_14985_amd import binding
    M, N, K = shape
    for dtype, transB in ((BF16, False), (FP16, True)):
        A, B = inputs.gemm_inputs(M, N, K, dtype, 11, transB=transB)
        bias = inputs.bias_input(N, dtype, 11, std=4.0) if with_bias else None
        binding.mlt_diag_force_variant(gemm=variant or "auto")
        st = pu.run_check_gemm_bias_act(A, B, bias, act, dtype, transB=transB)
        name = binding.mlt_last_kernel()
        print("   kernel=%s %s" % (name, st), flush=True)
        if with_bias or act:
            assert "skinny" not in name
        if variant in ("256pp16", "128pp16"):
            assert name.endswith("_pp16")


def test_fused_epilogue_edge_cases():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    # K = 0: C = act(bias)
    bias = torch.tensor([-2.0, 0.0, 3.0, -0.5, 1.5], dtype=torch.bfloat16, device=dev)
    A = torch.empty((4, 0), dtype=torch.bfloat16, device=dev)
    B = torch.empty((0, 5), dtype=torch.bfloat16, device=dev)
    C = binding.mlt_gemm_bias_act(A, B, bias, binding.ACT_RELU)
    torch.cuda.synchronize()
    assert torch.equal(C, torch.relu(bias).expand(4, 5))
    C = binding.mlt_gemm_bias_act(A, B, None, binding.ACT_GELU)
    torch.cuda.synchronize()
    assert torch.all(C == 0)
    # without bias and activation it is mlt_gemm, bit for bit
    A = torch.randn(300, 200, dtype=torch.float16, device=dev)
    B = torch.randn(200, 264, dtype=torch.float16, device=dev)
    assert torch.equal(binding.mlt_gemm_bias_act(A, B), binding.mlt_gemm(A, B))
    # errors: unknown activation, bias of the wrong length / dtype
    with pytest.raises(binding.MltError):
        binding.mlt_gemm_bias_act(A, B, None, 3)
    with pytest.raises(ValueError):
        binding.mlt_gemm_bias_act(A, B, torch.zeros(263, dtype=torch.float16, device=dev))
    with pytest.raises(ValueError):
        binding.mlt_gemm_bias_act(A, B, torch.zeros(264, dtype=torch.bfloat16, device=dev))


@pytest.mark.parametrize("tiling,tag", [(0, None), (1, "_w8x1"), (2, "_w1x8"), (3, "_w2x2")])
@pytest.mark.parametrize("transB", [False, True])
def test_tiling_hint(tiling, tag, transB):
    """The paper's tiling hint (Section 3.1): horizontal / vertical / square wave grids give the same
    C within the tolerance, from different kernels; several tiles, ragged edges, ragged and exact K."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    for dtype, (M, N, K) in ((BF16, (520, 776, 320)), (FP16, (300, 264, 200)), (BF16, (16, 2048, 512))):
        A, B = inputs.gemm_inputs(M, N, K, dtype, 13, transB=transB)
        tA = inputs.bits_to_torch(A, dtype, dev)
        tB = inputs.bits_to_torch(B, dtype, dev)
        C = binding.mlt_gemm_tiled(tA, tB, tiling, transB=transB)
        torch.cuda.synchronize()
        name = binding.mlt_last_kernel()
        st = pu.check_gemm(A, B, C, dtype, transB, seed=13)
        print("   kernel=%s %s" % (name, st), flush=True)
        if tag:
            # K % 64 != 0 takes the register-staged 2 x 2 kernel, else the pipelined one
            assert tag in name, name
    with pytest.raises(binding.MltError):
        binding.mlt_gemm_tiled(tA, tB, 4, transB=transB)
