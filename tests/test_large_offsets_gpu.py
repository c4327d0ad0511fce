"""GPU parity on problems whose tensors go beyond 2^31 elements / 4 GiB: every address the kernels
form for such a tensor has to be 64-bit arithmetic. Inputs that large are generated on the device
(torch generator, fixed seed); the oracle recomputes sampled outputs from the bit patterns copied
back for just those samples, chosen on both sides of the 2^31-byte, 2^32-byte and 2^31-element
offsets and at the far end."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2503_14985_amd import inputs
import parity_util as pu

pytestmark = pytest.mark.gpu
BF16, FP16 = inputs.BF16, inputs.FP16


@pytest.fixture(autouse=True)
def _announce(request):
    from paper_2503_14985_amd import binding
    print("\n[case] %s" % request.node.name, flush=True)
    binding.mlt_diag_force_variant(gemm="auto", mha="auto")
    yield
    binding.mlt_diag_force_variant(gemm="auto", mha="auto")
    torch.cuda.empty_cache()


def _gemm_samples(M, N, rng):
    """Whole rows around the row where the element offset passes 2^30, 2^31 (byte offsets 2^31,
    2^32), the first and last rows, plus random positions."""
    rows = {0, 1, M - 2, M - 1}
    for lim in (1 << 30, 1 << 31):
        r = lim // N
        rows.update(x for x in (r - 1, r, r + 1) if 0 <= x < M)
    rows = np.array(sorted(rows), dtype=np.int64)
    r = np.concatenate([np.repeat(rows, N), rng.integers(0, M, 200000)])
    c = np.concatenate([np.tile(np.arange(N), len(rows)), rng.integers(0, N, 200000)])
    return r, c


@pytest.mark.parametrize("variant", ["auto", "128pp16k128", "64k4"])
@pytest.mark.parametrize("transB", [False, True])
def test_gemm_output_beyond_2_31_elements(variant, transB):
    from paper_2503_14985_amd import binding
    M, N, K = 40960, 53248, 128                      # M * N = 2.18e9 elements, C is 4.4 GB
    assert M * N > 1 << 31
    A, B = inputs.gemm_inputs(M, N, K, BF16, 5, transB=transB)
    dev = torch.device("cuda:0")
    tA, tB = inputs.bits_to_torch(A, BF16, dev), inputs.bits_to_torch(B, BF16, dev)
    binding.mlt_diag_force_variant(gemm=variant)
    C = binding.mlt_gemm(tA, tB, transB=transB)
    torch.cuda.synchronize()
    print("   kernel=%s" % binding.mlt_last_kernel(), flush=True)
    assert bool(torch.isfinite(C).all())
    r, c = _gemm_samples(M, N, np.random.default_rng(11))
    got = C[torch.from_numpy(r).to(dev), torch.from_numpy(c).to(dev)].double().cpu().numpy()
    del C
    Bt = B if transB else np.ascontiguousarray(B.T)
    ref, T = oracle.gemm_sampled(A, Bt, r, c, BF16, transB=True)
    err = np.abs(got - ref)
    bound = pu.GEMM_TOL[BF16] * T + 1e-6
    assert np.all(err <= bound), "worst err/bound = %.3f" % float(np.max(err / bound))


@pytest.mark.parametrize("transB", [False, True])
def test_gemm_operand_rows_beyond_4_gib(transB):
    # A with a row stride of 65536 elements: its last rows start beyond 4 GiB (NaN in the padding)
    M, N, K = 40960, 512, 256
    A, B = inputs.gemm_inputs(M, N, K, BF16, 6, transB=transB)
    C = pu.run_gemm(A, B, BF16, transB=transB, lda=65536)
    st = pu.check_gemm(A, B, C, BF16, transB, seed=6)
    print("   %s" % st, flush=True)


def _device_normal(shape, dev, seed, dtype):
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    t = torch.empty(shape, device=dev, dtype=dtype)
    for b in range(shape[0]):                        # one batch entry at a time: no large temporaries
        t[b].normal_(generator=g)
    return t


@pytest.mark.parametrize("D,H,causal,dtype", [(128, 32, False, BF16), (64, 64, True, FP16)])
def test_attention_tensors_beyond_2_31_elements(D, H, causal, dtype):
    from paper_2503_14985_amd import binding
    B, S = 9, 65536                                  # B * H * S * D = 2.4e9 elements per tensor
    assert B * H * S * D > 1 << 31
    dev = torch.device("cuda:0")
    td = inputs.torch_dtype(dtype)
    Q = _device_normal((B, H, S, D), dev, 1, td)
    K = _device_normal((B, H, S, D), dev, 2, td)
    V = _device_normal((B, H, S, D), dev, 3, td)
    scale = 1.0 / math.sqrt(D)
    O = binding.mlt_mha_fwd(Q, K, V, scale=scale, causal=causal)
    torch.cuda.synchronize()
    print("   kernel=%s" % binding.mlt_last_kernel(), flush=True)
    head = S * D                                     # elements per (batch, head)
    picks = {0, B * H - 1}
    for lim in (1 << 30, 1 << 31):                   # heads on both sides of the offsets
        picks.update(x for x in (lim // head - 1, lim // head) if 0 <= x < B * H)
    rows = np.array([0, 255, 256, S // 2 + 31, S - 257, S - 1], dtype=np.int64)
    worst = 0.0
    for bh in sorted(picks):
        b, h = divmod(bh, H)
        qb = inputs.torch_to_bits(Q[b, h])[None, None]
        kb = inputs.torch_to_bits(K[b, h])[None, None]
        vb = inputs.torch_to_bits(V[b, h])[None, None]
        z = np.zeros(len(rows), dtype=np.int64)
        ref = oracle.mha_fwd_rows(qb, kb, vb, z, z, rows, scale, causal, dtype)
        got = O[b, h][torch.from_numpy(rows).to(dev)].double().cpu().numpy()
        assert np.all(np.isfinite(got))
        worst = max(worst, float(np.abs(got - ref).max()))
    print("   heads %s: max err %.3g" % (sorted(picks), worst), flush=True)
    assert worst <= pu.MHA_TOL[dtype]


def test_paged_cache_beyond_4_gib():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    Bp, Hp, Sp, Dp, bs = 80, 32, 8192, 128, 16       # K and V caches of 5.4 GB each
    nb = Bp * (Sp // bs)
    assert nb * Hp * bs * Dp > 1 << 31
    g = torch.Generator(device=dev)
    g.manual_seed(4)
    kc = _device_normal((nb, Hp, bs, Dp), dev, 7, torch.bfloat16)
    vc = _device_normal((nb, Hp, bs, Dp), dev, 8, torch.bfloat16)
    q = torch.randn((Bp, Hp, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    table = torch.randperm(nb, generator=g, device=dev).to(torch.int32).reshape(Bp, -1).contiguous()
    table[5, 0] = nb - 1                             # the last block of the cache is in use
    table[5, 1] = 0
    lens = torch.full((Bp,), Sp, dtype=torch.int32, device=dev)
    lens[7] = Sp - 37
    scale = 1.0 / math.sqrt(Dp)
    O = binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2)
    picks = [(5, 0), (5, Hp - 1), (7, 3), (0, 0), (Bp - 1, Hp - 1)] + \
            [(int(rng.integers(Bp)), int(rng.integers(Hp))) for _ in range(5)]
    worst = 0.0
    for b, h in picks:
        blocks = table[b].long()
        kb = inputs.torch_to_bits(kc[blocks, h].contiguous())[:, None]
        vb = inputs.torch_to_bits(vc[blocks, h].contiguous())[:, None]
        qb = inputs.torch_to_bits(q[b, h].contiguous())[None, None]
        t = np.arange(blocks.numel(), dtype=np.int32)[None]
        ref = oracle.paged_attn_decode(qb, kb, vb, t, np.array([int(lens[b])], np.int32), scale, BF16)
        worst = max(worst, float(np.abs(O[b, h].double().cpu().numpy() - ref[0, 0]).max()))
    print("   sampled max err %.3g" % worst, flush=True)
    assert worst <= pu.MHA_TOL[BF16]
