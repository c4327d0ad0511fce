"""GPU parity of mlt_mha_fwd against the fp64 oracle (through the C ABI via the ctypes binding)."""
import math
import os

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
    binding.mlt_diag_force_variant(mha="auto")
    binding.mlt_diag_set_persistent_grid(0)
    yield
    binding.mlt_diag_force_variant(mha="auto")
    binding.mlt_diag_set_persistent_grid(0)


def _go(B, H, Sq, Sk, D, dtype, causal, seed=0, scale=None, q_gain=1.0, **kw):
    from paper_2503_14985_amd import binding
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, dtype, seed, q_gain=q_gain)
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    O = pu.run_mha(Q, K, V, scale, causal, dtype)
    st = pu.check_mha(Q, K, V, O, scale, causal, dtype, seed=seed, **kw)
    print("   kernel=%s %s" % (binding.mlt_last_kernel(), st), flush=True)
    return st


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D", [64, 128])
def test_small_multi_tile(dtype, causal, D):
    # 2 query tiles of 256 and 5 key tiles of 64
    st = _go(1, 2, 512, 320, D, dtype, causal, seed=1)
    # sharper than the graded bound: output rounding plus P rounding only
    assert st["rel_rms"] < (1.5e-2 if dtype == BF16 else 2e-3)


@pytest.mark.parametrize("variant", ["pp16", "pp32", "ps"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D,dtype", [(128, BF16), (64, FP16), (128, FP16), (64, BF16)])
def test_every_kernel_variant(variant, causal, D, dtype):
    """The default is the two-group kernel on 32x32x16 MFMAs; its 16x16x32 form and the persistent
    form stay selectable and correct: several query and key tiles, ragged ends, peaky rows."""
    from paper_2503_14985_amd import binding
    # the persistent form exists for unmasked D = 128 only; elsewhere the request falls back to the
    # default kernel
    suffix = {"pp16": "_pp16", "pp32": "_pp", "ps": "_ps" if (D == 128 and not causal) else "_pp"}[variant]
    binding.mlt_diag_force_variant(mha=variant)
    _go(1, 2, 600, 455, D, dtype, causal, seed=11)
    assert binding.mlt_last_kernel().endswith(suffix)
    _go(2, 1, 300, 300, D, dtype, causal, seed=12, q_gain=3.0, rounding_aware=True)
    assert binding.mlt_last_kernel().endswith(suffix)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", ["ramp_up", "ramp_down", "spike_late"])
def test_reference_point_follows_the_scores(shape, dtype, D, causal):
    """Scores that change by far more than the lazy rescale's slack along the key axis: keys whose
    length grows (or shrinks) along the sequence, or one far-out key late in it. Growing scores
    make the kernel move its reference point many times, shrinking ones make later weights
    underflow (they are negligible then), the late spike makes one tile force a large move. The rows
    are peaky, hence the rounding-aware bound."""
    B, H, Sq, Sk = 1, 2, 320, 704
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, dtype, seed=21, q_gain=2.0)
    kf = pu.widen(K, dtype)
    pos = np.arange(Sk, dtype=np.float64)[None, None, :, None]
    if shape == "ramp_up":
        kf = kf * (0.25 + 6.0 * pos / Sk)
    elif shape == "ramp_down":
        kf = kf * (6.25 - 6.0 * pos / Sk)
    else:
        kf[:, :, 650, :] *= 12.0
    K = inputs.to_bits(kf.astype(np.float32), dtype)
    scale = 1.0 / math.sqrt(D)
    O = pu.run_mha(Q, K, V, scale, causal, dtype)
    st = pu.check_mha(Q, K, V, O, scale, causal, dtype, seed=21, rounding_aware=True)
    print("   %s" % st, flush=True)


@pytest.mark.parametrize("grid", [1, 3, 8, 0])
@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_persistent_kernel_walks_items(grid, dtype, D=128):
    """The unmasked case runs in the persistent kernel: every workgroup walks through several
    (head, query tile) items as one stream of key tiles. Few workgroups (the grid override) make
    each of them cross many item boundaries: 2 to 7 key tiles per item, ragged key and query ends
    (the last query tile of (3, 5, 300, .) leaves wavefronts without any row), a negative scale,
    peaky rows."""
    from paper_2503_14985_amd import binding
    binding.mlt_diag_force_variant(mha="ps")
    binding.mlt_diag_set_persistent_grid(grid)
    for (B, H, Sq, Sk, kw) in [(3, 5, 300, 200, {}), (1, 7, 700, 128, {}), (2, 3, 512, 435, {"q_gain": 3.0}),
                               (1, 9, 256, 100, {"scale": -0.11}), (1, 2, 1100, 65, {})]:
        _go(B, H, Sq, Sk, D, dtype, False, seed=31 + Sk, **kw)
        assert binding.mlt_last_kernel().endswith("_ps")
    # one key tile per item, and every masked problem, stay with the per-item kernel
    _go(1, 2, 300, 64, D, dtype, False, seed=5)
    assert binding.mlt_last_kernel().endswith("_pp")
    _go(1, 2, 300, 200, D, dtype, True, seed=6)
    assert binding.mlt_last_kernel().endswith("_pp")
    # D = 64 has no persistent form, forced or not
    _go(1, 2, 300, 200, 64, dtype, False, seed=9)
    assert binding.mlt_last_kernel().endswith("_pp")
    # the automatic choice never takes the persistent form
    binding.mlt_diag_force_variant(mha="auto")
    _go(1, 2, 300, 200, D, dtype, False, seed=7)
    assert binding.mlt_last_kernel().endswith("_pp")


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 1, 7, 1), (1, 3, 33, 17), (2, 2, 300, 200),
                                   (1, 2, 200, 300), (1, 1, 257, 65), (1, 1, 64, 1000)])
@pytest.mark.parametrize("causal", [False, True])
def test_ragged_shapes(shape, causal):
    B, H, Sq, Sk = shape
    _go(B, H, Sq, Sk, 128, BF16, causal, seed=2)
    _go(B, H, Sq, Sk, 64, FP16, causal, seed=2)


@pytest.mark.parametrize("causal", [False, True])
def test_peaky_scores_sharp_check(causal):
    """Q scaled x6: softmax concentrates, |O| ~ |V|, so the absolute bound bites."""
    st = _go(1, 2, 384, 384, 128, BF16, causal, seed=3, q_gain=6.0, rounding_aware=True)
    assert st["rel_rms"] < 1.5e-2
    st = _go(1, 2, 384, 384, 64, FP16, causal, seed=3, q_gain=6.0, rounding_aware=True)
    assert st["rel_rms"] < 2e-3


@pytest.mark.parametrize("scale", [0.0, -0.2, 1.0, 1e-3])
def test_scale_edge_values(scale):
    # scale = 1 makes the softmax peaky (|O| ~ |V|): see the rounding-aware bound
    _go(1, 2, 130, 190, 128, BF16, False, seed=4, scale=scale, rounding_aware=True)
    _go(1, 2, 130, 190, 64, BF16, True, seed=4, scale=scale, rounding_aware=True)


def test_structural_pins_on_gpu():
    """Q = 0 gives the mean of the visible V rows; causal row 0 is V[0]; constant V comes back."""
    B, H, S, D = 1, 2, 320, 128
    rng = np.random.default_rng(5)
    Q, K, V = inputs.mha_inputs(B, H, S, S, D, BF16, 5)
    Vd = pu.widen(V, BF16)
    Z = np.zeros_like(Q)
    O = pu.run_mha(Z, K, V, 0.3, False, BF16).double().cpu().numpy()
    assert np.max(np.abs(O - Vd.mean(axis=2, keepdims=True))) < 2e-3
    Oc = pu.run_mha(Z, K, V, 0.3, True, BF16).double().cpu().numpy()
    prefix = np.cumsum(Vd, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    assert np.max(np.abs(Oc - prefix)) < 1e-2
    Oc = pu.run_mha(Q, K, V, 0.3, True, BF16)
    assert np.array_equal(inputs.torch_to_bits(Oc)[:, :, 0, :], V[:, :, 0, :])   # row 0 = V[0] exactly
    v = inputs.to_bits(rng.standard_normal(D).astype(np.float32), BF16)
    Vc = np.broadcast_to(v, (B, H, S, D)).copy()
    Oc = pu.run_mha(Q, K, Vc, 0.3, False, BF16).double().cpu().numpy()
    assert np.max(np.abs(Oc - pu.widen(v, BF16)[None, None, None, :])) < 1.6e-2  # one bf16 ulp at |v|<4


def test_error_codes_on_gpu():
    from paper_2503_14985_amd import binding
    dev = torch.device("cuda:0")
    q = torch.zeros((1, 1, 4, 96), dtype=torch.bfloat16, device=dev)
    with pytest.raises(binding.MltError) as e:
        binding.mlt_mha_fwd(q, q, q, 1.0)
    assert e.value.status == binding.MLT_ERR_UNSUPPORTED
    q = torch.zeros((1, 1, 4, 64), dtype=torch.bfloat16, device=dev)
    k = torch.zeros((1, 1, 0, 64), dtype=torch.bfloat16, device=dev)
    with pytest.raises(binding.MltError) as e:
        binding.mlt_mha_fwd(q, k, k, 1.0)
    assert e.value.status == binding.MLT_ERR_INVALID_ARG
    o = binding.mlt_mha_fwd(q[:, :, :0], q, q, 1.0)       # Sq = 0: no-op
    assert o.shape == (1, 1, 0, 64)


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_config4_noncausal_full_size(dtype):
    st = _go(4, 32, 4096, 4096, 128, dtype, False, seed=0)
    assert st["rel_rms"] < (1.5e-2 if dtype == BF16 else 2e-3)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("S", [1024, 4096, 16384])
def test_config5_causal(S, D):
    _go(1, 32, S, S, D, BF16, True, seed=0, n_rows=512 if S <= 4096 else 160)


@pytest.mark.parametrize("H,D", [(32, 64), (16, 128)])
@pytest.mark.parametrize("causal", [False, True])
def test_paper_sweep_shape_fp16(H, D, causal):
    """One point of the paper's FlashAttention-2 sweep (Section 4.2: 32k tokens in total, hidden 2048
    as 32 heads x 64 or 16 heads x 128, fp16), here sequence 2048 x batch 16; sampled rows."""
    st = _go(16, H, 2048, 2048, D, FP16, causal, seed=0, n_rows=256)
    assert st["rel_rms"] < 2e-3


@pytest.mark.parametrize("H,D", [(32, 64), (16, 128)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("seq,batch,dtype", [(1024, 32, FP16), (32768, 1, FP16), (4096, 8, BF16), (32768, 1, BF16)])
def test_paper_sweep_ends_and_bf16_points(seq, batch, dtype, causal, H, D):
    """The ends of the paper's FlashAttention-2 sweep (Section 4.2): the shortest sequences (1024 x
    batch 32: the most workgroups, dominated by their first and last tiles) and the longest (32768 x
    batch 1: the most loop iterations and the largest K/V per head), both head layouts, causal and
    not, in fp16 as in the paper, and the bf16 points of this repository's table of the sweep.
    Sampled (batch, head, row) triples against all keys."""
    st = _go(batch, H, seq, seq, D, dtype, causal, seed=0, n_rows=48 if seq > 4096 else 96)
    assert st["rel_rms"] < (1.5e-2 if dtype == BF16 else 2e-3)
