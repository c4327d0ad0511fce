"""Pins for the CPU oracle: every check here compares it with something that is not itself.

Closed forms, textbook special cases, exact integer brute force, invariants of softmax attention
and library routines (torch float64 on the CPU). GEMM follows Section 2 / Listing 1 of
arXiv 2503.14985, attention follows Section 2.5, Algorithm 1. The paper prints no numeric
worked example for either, so there are no paper-value fixtures for these two functions; the
stored fixtures under tests/golden/ are small exact integer cases with their derivation.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2503_14985_amd import inputs

BF16, FP16 = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(x, dtype):
    return inputs.to_bits(np.asarray(x, dtype=np.float32), dtype)


def f64(b, dtype):
    """Independent widening through the library dtypes (not the oracle's converter)."""
    return inputs.bits_to_torch(b, dtype).double().numpy()


# ------------------------------------------------------------------------------- converters

def test_bf16_widen_exhaustive_vs_torch():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.to_f64(allb, BF16)
    want = f64(allb, BF16)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_f16_widen_exhaustive_vs_numpy():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.to_f64(allb, FP16)
    want = allb.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_widen_known_patterns():
    # values fixed by the formats themselves
    assert oracle.scalar_to_f64(0x3F80, BF16) == 1.0
    assert oracle.scalar_to_f64(0xC000, BF16) == -2.0
    assert oracle.scalar_to_f64(0x0001, BF16) == 2.0 ** -133       # smallest bf16 subnormal
    assert oracle.scalar_to_f64(0x3C00, FP16) == 1.0
    assert oracle.scalar_to_f64(0x0001, FP16) == 2.0 ** -24        # smallest fp16 subnormal
    assert oracle.scalar_to_f64(0x7BFF, FP16) == 65504.0           # largest finite fp16
    assert oracle.scalar_to_f64(0x0400, FP16) == 2.0 ** -14        # smallest fp16 normal


def _rne_fraction(x: Fraction, mant_bits: int, min_exp: int) -> Fraction:
    """Round-to-nearest-even of a positive rational onto a binary grid, in exact arithmetic."""
    e = 0
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    while Fraction(2) ** e > x:
        e -= 1
    e = max(e, min_exp)
    ulp = Fraction(2) ** (e - mant_bits)
    q = x / ulp
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl * ulp


@pytest.mark.parametrize("dtype,mant,min_exp", [(BF16, 7, -126), (FP16, 10, -14)])
def test_round_to_dtype_ties_and_random(dtype, mant, min_exp):
    ulp1 = Fraction(2) ** (-mant)
    cases = [1 + ulp1 / 2, 1 + 3 * ulp1 / 2, 1 + ulp1 / 2 + Fraction(1, 2 ** 40),
             1 + ulp1 / 2 - Fraction(1, 2 ** 40), Fraction(3, 7), Fraction(2) ** (min_exp - 3) * 5,
             Fraction(2) ** (min_exp) * (1 + ulp1 / 2)]
    rng = np.random.default_rng(5)
    cases += [Fraction(float(v)) for v in np.abs(rng.standard_normal(200)) * 3 + 1e-3]
    for x in cases:
        want = _rne_fraction(x, mant, min_exp)
        assert Fraction(oracle.round_to_dtype(float(x), dtype)) == want, x
        assert Fraction(oracle.round_to_dtype(-float(x), dtype)) == -want, x
    # ties-to-even examples spelled out
    if dtype == BF16:
        assert oracle.round_to_dtype(1 + 2.0 ** -8, BF16) == 1.0
        assert oracle.round_to_dtype(1 + 3 * 2.0 ** -8, BF16) == 1 + 2.0 ** -6


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_round_to_dtype_vs_torch_on_fp32_values(dtype):
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(2000) * np.exp(rng.uniform(-8, 8, 2000))).astype(np.float32)
    want = f64(inputs.to_bits(x, dtype), dtype)
    got = np.array([oracle.round_to_dtype(float(v), dtype) for v in x])
    assert np.array_equal(got, want)


# ------------------------------------------------------------------------------------- GEMM

def small_ints(rng, shape, lo=-4, hi=5):
    return rng.integers(lo, hi, size=shape).astype(np.float32)


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_gemm_identity_and_permutation_exact(dtype):
    rng = np.random.default_rng(0)
    n = 37
    a = rng.standard_normal((29, n)).astype(np.float32)
    A = bits(a, dtype)
    eye = bits(np.eye(n), dtype)
    C, T = oracle.gemm(A, eye, dtype)
    assert np.array_equal(C, f64(A, dtype))            # A * I = A exactly
    assert np.array_equal(T, np.abs(f64(A, dtype)))
    Bm = bits(rng.standard_normal((n, 23)), dtype)
    C2, _ = oracle.gemm(eye, Bm, dtype)
    assert np.array_equal(C2, f64(Bm, dtype))          # I * B = B exactly
    perm = rng.permutation(n)
    P = np.zeros((n, n), dtype=np.float32)
    P[np.arange(n), perm] = 1.0                        # row i of P*B is row perm[i] of B
    C3, _ = oracle.gemm(bits(P, dtype), Bm, dtype)
    assert np.array_equal(C3, f64(Bm, dtype)[perm])
    # a permutation on the right permutes columns: (A*P)[:, perm[i]] = A[:, i]
    C4, _ = oracle.gemm(A, bits(P, dtype), dtype)
    assert np.array_equal(C4[:, perm], f64(A, dtype))


def test_gemm_golden_4x4_integer_fixture():
    """Hand-sized integer case stored as text; expected product derived with exact integers."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gemm_4x4_int.txt"))
            if l.strip() and not l.startswith("#")]
    vals = np.array([[int(v) for v in r] for r in rows], dtype=np.int64)
    a, b, c = vals[0:4], vals[4:8], vals[8:12]
    # the fixture's third block is the integer product; verify with python ints (brute force)
    for i in range(4):
        for j in range(4):
            assert int(c[i, j]) == sum(int(a[i, k]) * int(b[k, j]) for k in range(4))
    for dtype in (BF16, FP16):
        C, T = oracle.gemm(bits(a, dtype), bits(b, dtype), dtype)
        assert np.array_equal(C, c.astype(np.float64))
        assert np.array_equal(T, (np.abs(a) @ np.abs(b)).astype(np.float64))
        # the transposed-storage path must see the same matrix
        Ct, _ = oracle.gemm(bits(a, dtype), bits(b.T.copy(), dtype), dtype, transB=True)
        assert np.array_equal(Ct, c.astype(np.float64))


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_gemm_integer_brute_force_rectangular(dtype):
    """Small-integer matrices: every product and partial sum is exact, so the oracle must equal
    exact integer arithmetic. Rectangular, so a swapped index or transposed operand fails."""
    rng = np.random.default_rng(1)
    M, N, K = 5, 7, 11
    a = small_ints(rng, (M, K))
    b = small_ints(rng, (K, N))
    want = np.array([[sum(int(a[i, k]) * int(b[k, j]) for k in range(K)) for j in range(N)]
                     for i in range(M)], dtype=np.float64)
    C, T = oracle.gemm(bits(a, dtype), bits(b, dtype), dtype)
    assert np.array_equal(C, want)
    wantT = np.array([[sum(abs(int(a[i, k])) * abs(int(b[k, j])) for k in range(K))
                       for j in range(N)] for i in range(M)], dtype=np.float64)
    assert np.array_equal(T, wantT)


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_gemm_closed_forms(dtype):
    M, N, K = 9, 13, 40
    ones_a = bits(np.ones((M, K)), dtype)
    ones_b = bits(np.ones((K, N)), dtype)
    C, T = oracle.gemm(ones_a, ones_b, dtype)
    assert np.all(C == K) and np.all(T == K)
    # a_ik = i, b_kj = j  =>  C_ij = K*i*j ; with alternating signs on k the sum telescopes
    a = np.repeat(np.arange(M, dtype=np.float32)[:, None], K, 1)
    b = np.repeat(np.arange(N, dtype=np.float32)[None, :], K, 0)
    C, T = oracle.gemm(bits(a, dtype), bits(b, dtype), dtype)
    want = K * np.outer(np.arange(M), np.arange(N)).astype(np.float64)
    assert np.array_equal(C, want) and np.array_equal(T, want)
    sign = np.where(np.arange(K) % 2 == 0, 1.0, -1.0).astype(np.float32)
    C, T = oracle.gemm(bits(a * sign[None, :], dtype), bits(b, dtype), dtype)
    assert np.all(C == 0.0) and np.array_equal(T, want)       # K even: cancels exactly
    # a_ik = k+1, b_kj = 1  =>  C_ij = K(K+1)/2 : depends on k actually running over all of K
    a = np.repeat(np.arange(1, K + 1, dtype=np.float32)[None, :], M, 0)
    C, _ = oracle.gemm(bits(a, dtype), ones_b, dtype)
    assert np.all(C == K * (K + 1) / 2)


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("shape", [(64, 48, 96), (130, 70, 257)])
def test_gemm_vs_torch_float64_matmul(dtype, shape):
    M, N, K = shape
    A, B = inputs.gemm_inputs(M, N, K, dtype, seed=3)
    C, T = oracle.gemm(A, B, dtype)
    ad, bd = f64(A, dtype), f64(B, dtype)
    want = torch.from_numpy(ad) @ torch.from_numpy(bd)
    wantT = torch.from_numpy(np.abs(ad)) @ torch.from_numpy(np.abs(bd))
    assert np.max(np.abs(C - want.numpy()) / wantT.numpy()) < 1e-14
    assert np.max(np.abs(T - wantT.numpy()) / wantT.numpy()) < 1e-14
    assert np.all(T >= np.abs(C))


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_gemm_transB_and_ld_and_sampled(dtype):
    M, N, K = 33, 21, 50
    A, B = inputs.gemm_inputs(M, N, K, dtype, seed=4)
    C, T = oracle.gemm(A, B, dtype)
    Ct, Tt = oracle.gemm(A, np.ascontiguousarray(B.T), dtype, transB=True)
    assert np.array_equal(C, Ct) and np.array_equal(T, Tt)            # bit for bit
    # padded leading dimensions (padding holds NaN patterns) change nothing
    Ap, Bp = inputs.gemm_inputs(M, N, K, dtype, seed=4, lda=K + 6, ldb=N + 10)
    assert Ap.strides[0] == 2 * (K + 6) and Bp.strides[0] == 2 * (N + 10)
    Cp, Tp = oracle.gemm(Ap, Bp, dtype)
    assert np.array_equal(C, Cp) and np.array_equal(T, Tp)
    rng = np.random.default_rng(9)
    r = rng.integers(0, M, 200)
    c = rng.integers(0, N, 200)
    Cs, Ts = oracle.gemm_sampled(A, B, r, c, dtype)
    assert np.array_equal(Cs, C[r, c]) and np.array_equal(Ts, T[r, c])
    Cs2, _ = oracle.gemm_sampled(A, np.ascontiguousarray(B.T), r, c, dtype, transB=True)
    assert np.array_equal(Cs2, C[r, c])


def test_gemm_edge_k0_and_single():
    A = np.zeros((3, 0), dtype=np.uint16)
    B = np.zeros((0, 4), dtype=np.uint16)
    C, T = oracle.gemm(A, B, BF16)
    assert C.shape == (3, 4) and np.all(C == 0) and np.all(T == 0)     # empty sum
    C, _ = oracle.gemm(bits([[3.0]], FP16), bits([[-0.5]], FP16), FP16)
    assert C[0, 0] == -1.5


# ---------------------------------------------------------------------------- fused epilogue

def test_epilogue_without_bias_and_activation_is_the_gemm():
    A, B = inputs.gemm_inputs(5, 7, 9, BF16, seed=21)
    C, T = oracle.gemm(A, B, BF16)
    Y, Ty = oracle.gemm_bias_act(A, B, None, oracle.ACT_NONE, BF16)
    assert np.array_equal(Y, C) and np.array_equal(Ty, T)


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_epilogue_bias_is_per_column_added_before_the_activation(dtype):
    # A = 0: the product vanishes and every ROW of the result is act(bias); 3 x 4, so a bias taken
    # by row, a subtracted bias or an activation applied before the bias all show
    A = np.zeros((3, 2), dtype=np.uint16)
    B = bits(np.ones((2, 4), dtype=np.float32), dtype)
    b = np.array([-1.0, 0.5, 2.0, -3.0])
    bias = bits(b.astype(np.float32), dtype)
    Y, T = oracle.gemm_bias_act(A, B, bias, oracle.ACT_NONE, dtype)
    assert np.array_equal(Y, np.tile(b, (3, 1)))
    assert np.array_equal(T, np.tile(np.abs(b), (3, 1)))          # the magnitude includes |bias|
    Y, _ = oracle.gemm_bias_act(A, B, bias, oracle.ACT_RELU, dtype)
    assert np.array_equal(Y, np.tile(np.maximum(b, 0.0), (3, 1)))


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_epilogue_integer_brute_force(dtype):
    rng = np.random.default_rng(22)
    a, b = small_ints(rng, (4, 6)), small_ints(rng, (6, 5))
    bias = small_ints(rng, (5,), -20, 20)
    want = [[sum(int(a[i, k]) * int(b[k, j]) for k in range(6)) + int(bias[j]) for j in range(5)]
            for i in range(4)]
    Y, _ = oracle.gemm_bias_act(bits(a, dtype), bits(b, dtype), bits(bias, dtype), oracle.ACT_NONE, dtype)
    assert np.array_equal(Y, np.array(want, dtype=np.float64))
    Y, _ = oracle.gemm_bias_act(bits(a, dtype), bits(b, dtype), bits(bias, dtype), oracle.ACT_RELU, dtype)
    assert np.array_equal(Y, np.maximum(np.array(want, dtype=np.float64), 0.0))
    Yt, _ = oracle.gemm_bias_act(bits(a, dtype), bits(b.T.copy(), dtype), bits(bias, dtype),
                                 oracle.ACT_RELU, dtype, transB=True)
    assert np.array_equal(Yt, Y)


def test_epilogue_gelu_against_the_normal_table_and_erfc():
    # x reaches the epilogue exactly as the 1 x 1 product 1 * x (+ bias 0 or with x split as
    # (x - 1) + bias 1)
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gelu_phi_table.txt"))
            if l.strip() and not l.startswith("#")]
    one = bits([[1.0]], FP16)
    for xs, phis in rows:
        x, phi = float(xs), float(phis)
        for sign in (1.0, -1.0):
            xv = sign * x
            ph = phi if sign > 0 else 1.0 - phi                   # Phi(-x) = 1 - Phi(x)
            Y, _ = oracle.gemm_bias_act(one, bits([[xv]], FP16), None, oracle.ACT_GELU, FP16)
            assert abs(Y[0, 0] - xv * ph) <= 4e-15 * max(1.0, abs(xv)), (xv, Y[0, 0])
            # the same value through the complementary error function (another libm routine)
            assert abs(Y[0, 0] - 0.5 * xv * math.erfc(-xv / math.sqrt(2.0))) <= 1e-15 * max(1.0, abs(xv))
            Y2, _ = oracle.gemm_bias_act(one, bits([[xv - 1.0]], FP16), bits([1.0], FP16),
                                         oracle.ACT_GELU, FP16)
            assert Y2[0, 0] == Y[0, 0]
    # far out: gelu(x) -> x and gelu(-x) -> -0
    Y, _ = oracle.gemm_bias_act(one, bits([[16.0]], FP16), None, oracle.ACT_GELU, FP16)
    assert Y[0, 0] == 16.0
    Y, _ = oracle.gemm_bias_act(one, bits([[-16.0]], FP16), None, oracle.ACT_GELU, FP16)
    assert abs(Y[0, 0]) < 1e-50


@pytest.mark.parametrize("act", [0, 1, 2])
def test_epilogue_vs_torch_float64_composition(act):
    A, B = inputs.gemm_inputs(9, 11, 33, BF16, seed=23)
    bias = inputs.to_bits(np.random.default_rng(24).standard_normal(11).astype(np.float32), BF16)
    Y, _ = oracle.gemm_bias_act(A, B, bias, act, BF16)
    x = torch.from_numpy(f64(A, BF16)) @ torch.from_numpy(f64(B, BF16)) + torch.from_numpy(f64(bias, BF16))
    want = [x, torch.relu(x), torch.nn.functional.gelu(x)][act].numpy()
    assert np.max(np.abs(Y - want)) <= 1e-13


# -------------------------------------------------------------------------------- attention

def torch_attention(q, k, v, scale, causal):
    """Library composition in float64: softmax(scale*QK^T + mask) V."""
    q, k, v = (torch.from_numpy(x) for x in (q, k, v))
    s = scale * q @ k.transpose(-1, -2)
    if causal:
        Sq, Sk = s.shape[-2:]
        mask = torch.arange(Sk)[None, :] > torch.arange(Sq)[:, None]
        s = s.masked_fill(mask, float("-inf"))
    return (torch.softmax(s, dim=-1) @ v).numpy()


@pytest.mark.parametrize("dtype", [BF16, FP16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 3, 17, 17, 8), (1, 2, 9, 30, 16), (1, 1, 30, 9, 4)])
def test_mha_vs_torch_float64(dtype, causal, shape):
    B, H, Sq, Sk, D = shape
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, dtype, seed=2)
    scale = 1.0 / math.sqrt(D)
    O = oracle.mha_fwd(Q, K, V, scale, causal, dtype)
    want = torch_attention(f64(Q, dtype), f64(K, dtype), f64(V, dtype), scale, causal)
    assert np.max(np.abs(O - want)) < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_mha_weights_sum_to_one_and_mask(causal):
    B, H, Sq, Sk, D = 1, 2, 12, 20, 8
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, BF16, seed=8)
    bs = np.zeros(Sq * H, dtype=np.int64)
    hs = np.repeat(np.arange(H), Sq)
    qs = np.tile(np.arange(Sq), H)
    O, W = oracle.mha_fwd_rows(Q, K, V, bs, hs, qs, 0.3, causal, BF16, want_weights=True)
    assert np.max(np.abs(W.sum(axis=1) - 1.0)) < 1e-15 * 8
    assert np.all(W >= 0)
    if causal:
        for r, i in enumerate(qs):
            assert np.all(W[r, i + 1:] == 0) and np.all(W[r, : i + 1] > 0)
    full = oracle.mha_fwd(Q, K, V, 0.3, causal, BF16)
    assert np.array_equal(O.reshape(H, Sq, D), full[0])
    # O is the weighted sum of V rows with exactly these weights
    vd = f64(V, BF16)
    for r in range(len(qs)):
        assert np.max(np.abs(W[r] @ vd[0, hs[r]] - O[r])) < 1e-14


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_mha_single_key_and_causal_row0(dtype):
    Q, K, V = inputs.mha_inputs(1, 2, 6, 1, 8, dtype, seed=1)
    O = oracle.mha_fwd(Q, K, V, 0.7, False, dtype)
    vd = f64(V, dtype)
    assert np.array_equal(O, np.broadcast_to(vd, O.shape))             # Sk = 1: O = V[0]
    Q, K, V = inputs.mha_inputs(2, 2, 7, 7, 8, dtype, seed=1)
    O = oracle.mha_fwd(Q, K, V, 0.7, True, dtype)
    assert np.array_equal(O[:, :, 0, :], f64(V, dtype)[:, :, 0, :])    # causal row 0 = V[0]
    # the last causal row sees every key: equals the unmasked result for that row
    On = oracle.mha_fwd(Q, K, V, 0.7, False, dtype)
    assert np.array_equal(O[:, :, -1, :], On[:, :, -1, :])
    assert not np.array_equal(O[:, :, 1, :], On[:, :, 1, :])


def test_mha_zero_query_gives_means():
    B, H, S, D = 1, 1, 6, 4
    _, K, V = inputs.mha_inputs(B, H, S, S, D, BF16, seed=6)
    Q = np.zeros((B, H, S, D), dtype=np.uint16)
    vd = f64(V, BF16)[0, 0]
    O = oracle.mha_fwd(Q, K, V, 1.0, False, BF16)[0, 0]
    assert np.max(np.abs(O - vd.mean(axis=0)[None, :])) < 1e-15        # uniform weights
    Oc = oracle.mha_fwd(Q, K, V, 1.0, True, BF16)[0, 0]
    for i in range(S):
        assert np.max(np.abs(Oc[i] - vd[: i + 1].mean(axis=0))) < 1e-15  # prefix mean
    # all V rows equal to v  =>  O = v up to rounding of the weights, for any Q (weights sum to 1, same addend)
    v = bits(np.array([0.5, -2.0, 3.0, 0.25]), BF16)
    Vc = np.broadcast_to(v, (B, H, S, D)).copy()
    Qr, _, _ = inputs.mha_inputs(B, H, S, S, D, BF16, seed=7)
    O2 = oracle.mha_fwd(Qr, K, Vc, 0.5, False, BF16)[0, 0]
    assert np.max(np.abs(O2 - f64(v, BF16)[None, :])) < 1e-14


def test_mha_two_key_closed_form_and_scale():
    """Two keys: the weights are the logistic function of the scaled score difference. A missing
    or squared scale, or a wrong sign in the exponent, changes the answer."""
    q = np.array([1.0, 2.0, -1.0, 0.5], dtype=np.float32)
    k = np.array([[0.5, -1.0, 2.0, 1.0], [1.5, 0.25, -0.5, 2.0]], dtype=np.float32)
    v = np.array([[1.0, 0.0, -2.0, 4.0], [-3.0, 2.0, 0.5, 1.0]], dtype=np.float32)
    scale = 0.35
    s0, s1 = float(q @ k[0]) * scale, float(q @ k[1]) * scale
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    want = w0 * v[0].astype(np.float64) + (1 - w0) * v[1].astype(np.float64)
    O = oracle.mha_fwd(bits(q, FP16).reshape(1, 1, 1, 4), bits(k, FP16).reshape(1, 1, 2, 4),
                       bits(v, FP16).reshape(1, 1, 2, 4), scale, False, FP16)
    assert np.max(np.abs(O[0, 0, 0] - want)) < 1e-15
    assert abs(s0 - s1) > 0.5      # the case does discriminate


def test_mha_shift_and_permutation_invariance():
    B, H, Sq, Sk, D = 1, 2, 5, 12, 8
    rng = np.random.default_rng(12)
    # small-integer-valued K and shift so that K+u is exactly representable
    q = bits(rng.standard_normal((B, H, Sq, D)), BF16)
    kf = small_ints(rng, (B, H, Sk, D))
    u = small_ints(rng, (D,))
    v = bits(rng.standard_normal((B, H, Sk, D)), BF16)
    O1 = oracle.mha_fwd(q, bits(kf, BF16), v, 0.25, False, BF16)
    O2 = oracle.mha_fwd(q, bits(kf + u, BF16), v, 0.25, False, BF16)
    assert np.max(np.abs(O1 - O2)) < 1e-12
    perm = rng.permutation(Sk)
    O3 = oracle.mha_fwd(q, bits(kf, BF16)[:, :, perm], v[:, :, perm], 0.25, False, BF16)
    assert np.max(np.abs(O1 - O3)) < 1e-13


def test_mha_one_hot_selects_value_row():
    S, D = 8, 8
    rng = np.random.default_rng(13)
    k = 64.0 * np.eye(S, D, dtype=np.float32)
    perm = rng.permutation(S)
    q = k[perm]
    v = rng.standard_normal((S, D)).astype(np.float32)
    V = bits(v, BF16).reshape(1, 1, S, D)
    O = oracle.mha_fwd(bits(q, BF16).reshape(1, 1, S, D), bits(k, BF16).reshape(1, 1, S, D), V,
                       1.0, False, BF16)[0, 0]
    # the matching key wins by 4096 in the exponent: weights are one-hot to machine precision
    assert np.max(np.abs(O - f64(V, BF16)[0, 0][perm])) < 1e-300 + 1e-15


def test_mha_head_and_batch_indexing():
    """Each (b, h) slice is an independent problem: the batched call equals per-slice calls."""
    B, H, Sq, Sk, D = 2, 3, 4, 6, 8
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, FP16, seed=21)
    O = oracle.mha_fwd(Q, K, V, 0.4, True, FP16)
    for b in range(B):
        for h in range(H):
            o = oracle.mha_fwd(Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], 0.4,
                               True, FP16)
            assert np.array_equal(o[0, 0], O[b, h])


def test_blockwise_online_softmax_equals_plain_oracle():
    """The tiled recurrence the GPU kernel uses (running max m, running sum l, rescaled O, final
    division; Algorithm 1 with the rescale written out) is the same function as the plain
    softmax the oracle evaluates. Written here in float64, never in the oracle."""
    B, H, Sq, Sk, D = 1, 1, 7, 45, 8
    Q, K, V = inputs.mha_inputs(B, H, Sq, Sk, D, BF16, seed=30)
    qd, kd, vd = f64(Q, BF16)[0, 0], f64(K, BF16)[0, 0], f64(V, BF16)[0, 0]
    scale = 0.3
    for causal in (False, True):
        want = oracle.mha_fwd(Q, K, V, scale, causal, BF16)[0, 0]
        for block in (1, 4, 16, 64):
            m = np.full(Sq, -np.inf)
            l = np.zeros(Sq)
            o = np.zeros((Sq, D))
            for j0 in range(0, Sk, block):
                s = scale * qd @ kd[j0:j0 + block].T
                if causal:
                    jj = np.arange(j0, min(j0 + block, Sk))
                    s = np.where(jj[None, :] <= np.arange(Sq)[:, None], s, -np.inf)
                m_new = np.maximum(m, s.max(axis=1))
                alpha = np.where(np.isinf(m_new), 1.0, np.exp(m - m_new))
                p = np.where(np.isinf(m_new)[:, None], 0.0, np.exp(s - m_new[:, None]))
                l = alpha * l + p.sum(axis=1)
                o = alpha[:, None] * o + p @ vd[j0:j0 + block]
                m = m_new
            assert np.max(np.abs(o / l[:, None] - want)) < 1e-13


# ------------------------------------------------------------------ paged attention (decoding)

def _paged_case(dtype=BF16, seed=11, poison=False, shuffle=True):
    from paper_2503_14985_amd import inputs
    lens = [1, 5, 16, 17, 40]
    return inputs.paged_inputs(len(lens), 3, 32, 8, lens, dtype, seed, shuffle=shuffle, poison=poison)


@pytest.mark.parametrize("dtype", [BF16, FP16])
def test_paged_equals_dense_attention_on_the_gathered_keys(dtype):
    """With the logical keys gathered, decoding is the last-row case of the (separately pinned)
    dense attention oracle: one query over seq_len keys, no mask."""
    q, kc, vc, table, lens, kd, vd = _paged_case(dtype)
    O = oracle.paged_attn_decode(q, kc, vc, table, lens, 0.37, dtype)
    for b in range(q.shape[0]):
        dense = oracle.mha_fwd(q[b][None, :, None, :], kd[b][None], vd[b][None], 0.37, False, dtype)
        assert np.array_equal(O[b], dense[0, :, 0, :])


def test_paged_matches_torch_float64_composition():
    import torch
    q, kc, vc, table, lens, kd, vd = _paged_case(BF16, seed=12)
    O, W = oracle.paged_attn_decode(q, kc, vc, table, lens, 0.5, BF16, want_weights=True)
    for b in range(q.shape[0]):
        qt = torch.from_numpy(oracle.to_f64(q[b], BF16))                   # [H, D]
        kt = torch.from_numpy(oracle.to_f64(kd[b], BF16))                  # [H, n, D]
        vt = torch.from_numpy(oracle.to_f64(vd[b], BF16))
        w = torch.softmax(0.5 * torch.einsum("hd,hnd->hn", qt, kt), dim=-1)
        ref = torch.einsum("hn,hnd->hd", w, vt).numpy()
        assert np.max(np.abs(O[b] - ref)) < 1e-12
        n = int(lens[b])
        assert np.max(np.abs(W[b, :, :n] - w.numpy())) < 1e-13
        assert np.all(W[b, :, n:] == 0.0)
        assert np.max(np.abs(W[b].sum(axis=-1) - 1.0)) < 1e-14


def test_paged_block_placement_is_irrelevant_and_unused_storage_is_never_read():
    a = _paged_case(BF16, seed=13, shuffle=False)
    b = _paged_case(BF16, seed=13, shuffle=True, poison=True)
    # same draws (the permutation is drawn first only when shuffling, so compare through the
    # dense keys): the two caches hold the same logical sequences
    qa, kca, vca, ta, la, kda, vda = a
    from paper_2503_14985_amd import inputs
    # rebuild b's cache from a's logical data in b's (shuffled, poisoned) block order
    qb, kcb, vcb, tb, lb, _, _ = b
    bs = kcb.shape[2]
    for s in range(qa.shape[0]):
        n = int(la[s])
        for i in range((n + bs - 1) // bs):
            lo, hi = i * bs, min((i + 1) * bs, n)
            kcb[tb[s, i], :, : hi - lo] = kda[s][:, lo:hi]
            vcb[tb[s, i], :, : hi - lo] = vda[s][:, lo:hi]
    Oa = oracle.paged_attn_decode(qa, kca, vca, ta, la, 0.21, BF16)
    Ob = oracle.paged_attn_decode(qa, kcb, vcb, tb, la, 0.21, BF16)
    assert np.all(np.isfinite(Ob))
    assert np.array_equal(Oa, Ob)


def test_paged_single_key_two_keys_and_constant_values():
    from paper_2503_14985_amd import inputs
    q, kc, vc, table, lens, kd, vd = inputs.paged_inputs(2, 2, 16, 4, [1, 2], BF16, 14)
    O, W = oracle.paged_attn_decode(q, kc, vc, table, lens, 0.8, BF16, want_weights=True)
    assert np.array_equal(O[0], oracle.to_f64(vd[0][:, 0, :], BF16))           # one key: O = V[0]
    qd, k2 = oracle.to_f64(q[1], BF16), oracle.to_f64(kd[1], BF16)
    s = 0.8 * np.einsum("hd,hnd->hn", qd, k2)
    w0 = 1.0 / (1.0 + np.exp(s[:, 1] - s[:, 0]))                               # logistic closed form
    assert np.max(np.abs(W[1, :, 0] - w0)) < 1e-14
    # constant values come back whatever the weights are
    vc2 = np.empty_like(vc)
    vc2[:] = inputs.to_bits(np.full((1,), 1.5, np.float32), BF16)[0]
    O2 = oracle.paged_attn_decode(q, kc, vc2, table, lens, 0.8, BF16)
    assert np.max(np.abs(O2 - 1.5)) < 1e-14


def test_paged_heads_and_sequences_are_independent():
    q, kc, vc, table, lens, kd, vd = _paged_case(FP16, seed=15)
    O = oracle.paged_attn_decode(q, kc, vc, table, lens, 0.3, FP16)
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[:, 1] ^= 0x0155                      # disturb head 1 everywhere
    vc2[:, 1] ^= 0x0155
    O2 = oracle.paged_attn_decode(q, kc2, vc2, table, lens, 0.3, FP16)
    assert np.array_equal(O[:, [0, 2]], O2[:, [0, 2]]) and not np.array_equal(O[:, 1], O2[:, 1])
    # swapping two sequences' rows of the table and lengths swaps their outputs
    t2, l2, q2 = table.copy(), lens.copy(), q.copy()
    t2[[1, 3]] = t2[[3, 1]]; l2[[1, 3]] = l2[[3, 1]]; q2[[1, 3]] = q2[[3, 1]]
    O3 = oracle.paged_attn_decode(q2, kc, vc, t2, l2, 0.3, FP16)
    assert np.array_equal(O3[[1, 3]], O[[3, 1]]) and np.array_equal(O3[[0, 2, 4]], O[[0, 2, 4]])


def test_paged_rejects_bad_tables_and_lengths():
    q, kc, vc, table, lens, _, _ = _paged_case(BF16, seed=16)
    bad = table.copy(); bad[4, 0] = kc.shape[0]
    with pytest.raises(RuntimeError):
        oracle.paged_attn_decode(q, kc, vc, bad, lens, 1.0, BF16)
    l0 = lens.copy(); l0[2] = 0
    with pytest.raises(RuntimeError):
        oracle.paged_attn_decode(q, kc, vc, table, l0, 1.0, BF16)
