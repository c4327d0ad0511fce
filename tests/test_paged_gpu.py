"""GPU parity of mlt_paged_attn_decode against the fp64 oracle (through the C ABI)."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2503_14985_amd import inputs

pytestmark = pytest.mark.gpu
BF16, FP16 = inputs.BF16, inputs.FP16
# the attention tolerances of the benchmark spec (absolute, on O), plus a relative-RMS check
TOL = {BF16: 1e-2, FP16: 2e-3}
RMS = {BF16: 1.5e-2, FP16: 2e-3}


@pytest.fixture(autouse=True)
def _announce(request):
    print("\n[case] %s" % request.node.name, flush=True)
    yield


def _run(q, kc, vc, table, lens, scale, dtype):
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    Q, Kc, Vc = (inputs.bits_to_torch(x, dtype, dev) for x in (q, kc, vc))
    T = torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).to(dev)
    L = torch.from_numpy(np.ascontiguousarray(lens, dtype=np.int32)).to(dev)
    O = binding.mlt_paged_attn_decode(Q, Kc, Vc, T, L, scale)
    torch.cuda.synchronize()
    return O


def _check(B, H, D, bs, lens, dtype, seed, scale=None, poison=True):
    from paper_2503_14985_amd import binding
    q, kc, vc, table, lens, _, _ = inputs.paged_inputs(B, H, D, bs, lens, dtype, seed, poison=poison)
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    O = _run(q, kc, vc, table, lens, scale, dtype)
    Og = O.double().cpu().numpy()
    assert np.all(np.isfinite(Og)), "non-finite output"
    # the oracle refuses out-of-range table entries: give it the table with the unused entries zeroed
    t = table.copy()
    t[t >= kc.shape[0]] = 0
    Oref = oracle.paged_attn_decode(q, kc, vc, t, lens, scale, dtype)
    err = np.abs(Og - Oref)
    rel = float(np.sqrt(np.mean(err ** 2)) / max(np.sqrt(np.mean(Oref ** 2)), 1e-30))
    print("   kernel=%s max err %.3g rel rms %.3g" % (binding.mlt_last_kernel(), err.max(), rel), flush=True)
    assert err.max() <= TOL[dtype], "paged attention parity: max err %.3g" % err.max()
    assert rel <= RMS[dtype], "paged attention parity: rel rms %.3g" % rel
    return Og, Oref


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("bs", [16, 64])
def test_ragged_lengths(dtype, D, bs):
    # lengths around unit (16), block and wavefront-split boundaries, incl. 1 and a full table
    lens = [1, 2, 15, 16, 17, 63, 64, 65, 100, 257, 1000, 4 * bs]
    _check(len(lens), 3, D, bs, lens, dtype, seed=1)


def test_long_sequences_bf16():
    _check(4, 8, 128, 16, [4096, 3001, 8192, 77], BF16, seed=2)


@pytest.mark.parametrize("scale", [0.0, -0.3, 1.0])
def test_scale_edge_values(scale):
    _check(3, 2, 128, 32, [5, 130, 700], BF16, seed=3, scale=scale)
    _check(3, 2, 64, 32, [5, 130, 700], FP16, seed=3, scale=scale)


def test_structure_single_key_and_constant_values():
    from paper_2503_14985_amd import binding
    q, kc, vc, table, lens, kd, vd = inputs.paged_inputs(3, 4, 128, 16, [1, 33, 200], BF16, 4)
    O = _run(q, kc, vc, table, lens, 0.2, BF16)
    assert np.array_equal(inputs.torch_to_bits(O)[0], vd[0][:, 0, :])          # one key: O = V[0] exactly
    vc2 = np.empty_like(vc)
    vc2[:] = inputs.to_bits(np.full((1,), -2.5, np.float32), BF16)[0]
    O2 = _run(q, kc, vc2, table, lens, 0.2, BF16).double().cpu().numpy()
    assert np.max(np.abs(O2 + 2.5)) <= 2.5 * 2.0 ** -8                         # constant V comes back
    # block placement is irrelevant: the same logical data in another physical order -> same bits
    perm = np.random.default_rng(9).permutation(kc.shape[0])
    inv = np.argsort(perm)
    kc3, vc3 = kc[perm], vc[perm]                # physical block i now holds old block perm[i]
    table3 = inv[table].astype(np.int32)         # ... so old block j is found at inv[j]
    O3 = _run(q, kc3, vc3, table3, lens, 0.2, BF16)
    assert torch.equal(O3, O)


def test_bad_table_entries_are_clamped_not_followed():
    """Entries outside the cache must not fault: the result for that sequence is unspecified but
    finite inputs stay finite and the other sequences are unaffected."""
    q, kc, vc, table, lens, _, _ = inputs.paged_inputs(3, 2, 64, 16, [40, 40, 40], BF16, 5, poison=False)
    good = _run(q, kc, vc, table, lens, 0.1, BF16)
    bad = table.copy()
    bad[1, 1] = 10 ** 6
    bad[1, 2] = -5
    out = _run(q, kc, vc, bad, lens, 0.1, BF16)
    assert torch.equal(out[[0, 2]], good[[0, 2]]) and bool(torch.isfinite(out.float()).all())


def test_argument_errors():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    q = torch.zeros(2, 2, 96, dtype=torch.bfloat16, device=dev)
    kc = torch.zeros(4, 2, 16, 96, dtype=torch.bfloat16, device=dev)
    t = torch.zeros(2, 2, dtype=torch.int32, device=dev)
    l = torch.ones(2, dtype=torch.int32, device=dev)
    with pytest.raises(binding.MltError) as e:
        binding.mlt_paged_attn_decode(q, kc, kc, t, l, 1.0)
    assert e.value.status == binding.MLT_ERR_UNSUPPORTED                       # D = 96
    q = torch.zeros(2, 2, 64, dtype=torch.bfloat16, device=dev)
    kc = torch.zeros(4, 2, 24, 64, dtype=torch.bfloat16, device=dev)
    with pytest.raises(binding.MltError) as e:
        binding.mlt_paged_attn_decode(q, kc, kc, t, l, 1.0)
    assert e.value.status == binding.MLT_ERR_UNSUPPORTED                       # block_size = 24
    kc = torch.zeros(4, 2, 16, 64, dtype=torch.bfloat16, device=dev)
    with pytest.raises(binding.MltError) as e:
        binding.mlt_paged_attn_decode(q, kc, kc, t, l, float("nan"))
    assert e.value.status == binding.MLT_ERR_INVALID_ARG


def test_bench_size_sampled_heads():
    """The bench workload (64 sequences x 32 heads x 4096 keys, shuffled 16-key blocks), generated
    on the device; the oracle recomputes 12 sampled (sequence, head) outputs from their blocks."""
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    Bp, Hp, Sp, Dp, bs = 64, 32, 4096, 128, 16
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    nb = Bp * (Sp // bs)
    kc = torch.randn((nb, Hp, bs, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    vc = torch.randn((nb, Hp, bs, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    q = torch.randn((Bp, Hp, Dp), generator=g, device=dev, dtype=torch.bfloat16)
    table = torch.randperm(nb, generator=g, device=dev).to(torch.int32).reshape(Bp, -1).contiguous()
    lens = torch.full((Bp,), Sp, dtype=torch.int32, device=dev)
    lens[3] = 4001                                          # one ragged sequence among the samples
    scale = 1.0 / math.sqrt(Dp)
    O = binding.mlt_paged_attn_decode(q, kc, vc, table, lens, scale)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    picks = [(3, 0), (0, 0), (Bp - 1, Hp - 1)] + [(int(rng.integers(Bp)), int(rng.integers(Hp))) for _ in range(9)]
    worst = 0.0
    for b, h in picks:
        blocks = table[b].long()
        kb = inputs.torch_to_bits(kc[blocks, h].contiguous().cpu())[:, None]      # [nblk, 1, bs, D]
        vb = inputs.torch_to_bits(vc[blocks, h].contiguous().cpu())[:, None]
        qb = inputs.torch_to_bits(q[b, h].contiguous().cpu())[None, None]         # [1, 1, D]
        t = np.arange(blocks.numel(), dtype=np.int32)[None]
        ref = oracle.paged_attn_decode(qb, kb, vb, t, np.array([int(lens[b])], np.int32), scale, BF16)
        err = np.abs(O[b, h].double().cpu().numpy() - ref[0, 0]).max()
        worst = max(worst, float(err))
    print("   sampled max err %.3g" % worst, flush=True)
    assert worst <= TOL[BF16]


@pytest.fixture
def key_split():
    """Forces the number of key ranges per (sequence, head) for one test, then restores the
    library's own choice."""
    from paper_2503_14985_amd import binding
    yield binding.mlt_diag_force_key_split
    binding.mlt_diag_force_key_split(0)


@pytest.mark.parametrize("nsplit", [2, 3, 7, 64])
@pytest.mark.parametrize("dtype,D", [(BF16, 128), (FP16, 64)])
def test_key_split_across_workgroups(key_split, nsplit, dtype, D):
    """Keys cut into ranges over several workgroups, merged by the second kernel: lengths from one
    key (every range but the first empty) to ranges that end inside a unit, a block and a wavefront
    round."""
    from paper_2503_14985_amd import binding
    key_split(nsplit)
    lens = [1, 2, 16, 17, 63, 65, 100, 257, 1000, 1023, 2048, 3001]
    _check(len(lens), 3, D, 16, lens, dtype, seed=11)
    assert binding.mlt_last_kernel().endswith("_keysplit%d" % nsplit)
    _check(2, 2, D, 64, [4096, 777], dtype, seed=12)


def test_key_split_is_chosen_for_few_long_sequences_and_repeats_bit_for_bit(key_split):
    from paper_2503_14985_amd import binding
    key_split(0)
    q, kc, vc, table, lens, _, _ = inputs.paged_inputs(2, 4, 128, 16, [16384, 9000], BF16, 13)
    scale = 1.0 / math.sqrt(128)
    O1 = _run(q, kc, vc, table, lens, scale, BF16)
    assert "_keysplit" in binding.mlt_last_kernel(), binding.mlt_last_kernel()
    O2 = _run(q, kc, vc, table, lens, scale, BF16)
    assert torch.equal(O1, O2)                              # fixed merge order: no run-to-run change
    t = table.copy()
    t[t >= kc.shape[0]] = 0
    ref = oracle.paged_attn_decode(q, kc, vc, t, lens, scale, BF16)
    assert np.abs(O1.double().cpu().numpy() - ref).max() <= TOL[BF16]
    # many pairs: the plain form
    _check(40, 32, 128, 16, [100] * 40, BF16, seed=14)
    assert "_keysplit" not in binding.mlt_last_kernel()


def test_key_split_single_key_and_block_placement(key_split):
    key_split(5)
    q, kc, vc, table, lens, kd, vd = inputs.paged_inputs(3, 4, 128, 16, [1, 33, 2000], BF16, 4)
    O = _run(q, kc, vc, table, lens, 0.2, BF16)
    assert np.array_equal(inputs.torch_to_bits(O)[0], vd[0][:, 0, :])          # one key: O = V[0] exactly
    perm = np.random.default_rng(9).permutation(kc.shape[0])
    inv = np.argsort(perm)
    O3 = _run(q, kc[perm], vc[perm], inv[table].astype(np.int32), lens, 0.2, BF16)
    assert torch.equal(O3, O)
