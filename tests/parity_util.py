"""Helpers for the GPU parity tests: run the HIP path through the binding, run the oracle on the
same 16-bit patterns, compare with the stated tolerances."""
import numpy as np
import torch

import oracle
from paper_2503_14985_amd import inputs

GEMM_TOL = {inputs.BF16: 8e-3, inputs.FP16: 1e-3}       # |C - C_ref| <= tol * (|A||B|) + 1e-6
MHA_TOL = {inputs.BF16: 1e-2, inputs.FP16: 2e-3}        # max |O - O_ref|


def widen(bits, dtype):
    """16-bit patterns -> float64 through the library dtype (exact)."""
    return inputs.bits_to_torch(bits, dtype).double().numpy()


def gemm_seam_samples(M, N, rng, tile=256, sub=32, nrand=65536, nlines=16):
    """Positions for the sampled check: whole rows and columns on both sides of tile and
    wavefront seams (and the first/last), plus uniformly random positions."""
    def lines(n):
        cand = {0, n - 1}
        for s in (sub, 2 * sub, tile // 2, tile):
            for b in (s - 1, s, n - s - 1, n - s):
                if 0 <= b < n:
                    cand.add(b)
        cand = sorted(cand)
        if len(cand) > nlines:
            keep = {0, n - 1}
            rest = [c for c in cand if c not in keep]
            pick = rng.choice(len(rest), nlines - 2, replace=False)
            cand = sorted(keep | {rest[i] for i in pick})
        return np.array(cand, dtype=np.int64)
    rws, cls = lines(M), lines(N)
    r = [np.repeat(rws, N), np.tile(np.arange(M), len(cls)), rng.integers(0, M, nrand)]
    c = [np.tile(np.arange(N), len(rws)), np.repeat(cls, M), rng.integers(0, N, nrand)]
    return np.concatenate(r), np.concatenate(c)


def check_gemm(A, B, C_gpu, dtype, transB, full_limit=1 << 28, seed=0):
    """A, B: uint16 patterns (B is [N,K] when transB). C_gpu: torch tensor [M,N] from the HIP path.
    Full oracle when M*N*K is small, seam + random samples otherwise. Returns stats."""
    M, K = A.shape
    N = B.shape[0] if transB else B.shape[1]
    Cg = C_gpu.detach().cpu().double().numpy()
    assert Cg.shape == (M, N)
    tol = GEMM_TOL[dtype]
    if M * N * max(K, 1) <= full_limit:
        Cref, T = oracle.gemm(A, B, dtype, transB=transB)
        err = np.abs(Cg - Cref)
        bound = tol * T + 1e-6
    else:
        rng = np.random.default_rng(seed + 12345)
        r, c = gemm_seam_samples(M, N, rng)
        # k-contiguous copy of B for the oracle's inner loop (same matrix, other storage order)
        Bt = B if transB else np.ascontiguousarray(B.T)
        Cref, T = oracle.gemm_sampled(A, Bt, r, c, dtype, transB=True)
        err = np.abs(Cg[r, c] - Cref)
        bound = tol * T + 1e-6
    worst = float(np.max(err / bound)) if err.size else 0.0
    assert np.all(np.isfinite(Cg)), "non-finite output"
    assert np.all(err <= bound), "GEMM parity: worst err/bound = %.3f, max err %.3g" % (worst, err.max())
    return {"max_err": float(err.max()) if err.size else 0.0, "worst_ratio": worst, "n": int(err.size)}


def _device_matrix(bits, dtype, dev, ld=None):
    """Upload a matrix; with ld > columns it becomes a row-strided view into a NaN-filled buffer."""
    t = inputs.bits_to_torch(np.ascontiguousarray(bits), dtype, dev)
    if ld is None or ld == bits.shape[1]:
        return t
    buf = torch.full((bits.shape[0], ld), float("nan"), dtype=t.dtype, device=dev)
    buf[:, : bits.shape[1]] = t
    return buf[:, : bits.shape[1]]


def run_gemm(A, B, dtype, transB=False, device="cuda:0", lda=None, ldb=None, ldc_pad=0):
    from paper_2503_14985_amd import binding
    dev = torch.device(device)
    tA = _device_matrix(A, dtype, dev, lda)
    tB = _device_matrix(B, dtype, dev, ldb)
    C = None
    M = A.shape[0]
    N = B.shape[0] if transB else B.shape[1]
    if ldc_pad:
        buf = torch.full((M, N + ldc_pad), float("nan"), dtype=tA.dtype, device=dev)
        C = buf[:, :N]
    out = binding.mlt_gemm(tA, tB, C=C, transB=transB)
    torch.cuda.synchronize()
    if ldc_pad:
        assert torch.isnan(buf[:, N:]).all(), "kernel wrote into the padding of C"
    return out


# Fused epilogue: y = act(x + bias). The activation has Lipschitz constant 1 (none, ReLU) or
# max |gelu'| = 1.129 (GELU), so an error e in x + bias becomes at most 1.13 * e; the final rounding to
# 16 bit is relative to |y| <= |x + bias| <= T + |bias|, which the GEMM tolerance (four rounding units
# of the output type) covers as it does for the plain GEMM.
ACT_LIPSCHITZ = {0: 1.0, 1: 1.0, 2: 1.13}


def run_check_gemm_bias_act(A, B, bias, act, dtype, transB=False, device="cuda:0"):
    from paper_2503_14985_amd import binding
    dev = torch.device(device)
    tA = inputs.bits_to_torch(np.ascontiguousarray(A), dtype, dev)
    tB = inputs.bits_to_torch(np.ascontiguousarray(B), dtype, dev)
    tb = inputs.bits_to_torch(bias, dtype, dev) if bias is not None else None
    M = A.shape[0]
    N = B.shape[0] if transB else B.shape[1]
    buf = torch.full((M, N + 3), float("nan"), dtype=tA.dtype, device=dev)
    out = binding.mlt_gemm_bias_act(tA, tB, tb, act, C=buf[:, :N], transB=transB)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, N:]).all(), "kernel wrote into the padding of C"
    Yg = out.detach().cpu().double().numpy()
    Yref, T = oracle.gemm_bias_act(A, B, bias, act, dtype, transB=transB)
    err = np.abs(Yg - Yref)
    bound = ACT_LIPSCHITZ[act] * GEMM_TOL[dtype] * T + 1e-6
    worst = float(np.max(err / bound)) if err.size else 0.0
    assert np.all(np.isfinite(Yg)), "non-finite output"
    assert np.all(err <= bound), "fused GEMM parity: worst err/bound = %.3f, max err %.3g" % (worst, err.max())
    return {"max_err": float(err.max()) if err.size else 0.0, "worst_ratio": worst, "n": int(err.size)}


def mha_sample_rows(B, H, Sq, rng, n_bh=8, n_rows=512, tile=128, wave=32):
    """(batch, head, query row) samples: first and last heads plus random ones; for each the first
    rows, the last row, both sides of workgroup-tile seams and of wavefront seams (every `wave`
    rows: all of them while they fit a quarter of the budget, else a random choice), the rest random."""
    bh = {(0, 0), (B - 1, H - 1)}
    while len(bh) < min(n_bh, B * H):
        bh.add((int(rng.integers(0, B)), int(rng.integers(0, H))))
    rows = {0, 1, 2, 3, Sq - 1}
    for t in range(tile, Sq, tile):
        rows.update((t - 1, t))
        if len(rows) > n_rows // 2:
            break
    seams = np.arange(wave, Sq, wave)
    seams = seams[seams % tile != 0]
    budget = max(2, n_rows // 8)
    if len(seams) > budget:
        seams = rng.choice(seams, budget, replace=False)
    for t in seams:
        rows.update((int(t) - 1, int(t)))
    rows = sorted(r for r in rows if 0 <= r < Sq)
    bs, hs, qs = [], [], []
    for (b, h) in sorted(bh):
        extra = rng.integers(0, Sq, max(0, n_rows - len(rows)))
        for r in list(rows) + list(extra):
            bs.append(b); hs.append(h); qs.append(int(r))
    return np.array(bs), np.array(hs), np.array(qs)


def round_to_dtype(x, dtype):
    """fp64 array -> nearest value of the 16-bit type, ties to even, computed in fp64 (a cast through
    fp32 would round twice). Finite values inside the type's range only."""
    sig_bits = 8 if dtype == inputs.BF16 else 11          # significand bits, hidden bit included
    min_exp = -126 if dtype == inputs.BF16 else -14
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                                     # |x| = m * 2^e with 0.5 <= m < 1
    q = np.exp2(np.maximum(e, min_exp + 1) - sig_bits)     # spacing at x (subnormals: the smallest)
    return np.rint(x / q) * q


def ulp_of(x, dtype):
    """Spacing of the 16-bit type at |x| (normal range; the smallest normal's spacing below it)."""
    frac_bits = 7 if dtype == inputs.BF16 else 10
    min_exp = -126 if dtype == inputs.BF16 else -14
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** min_exp)))
    return 2.0 ** (e - frac_bits)


def check_mha(Q, K, V, O_gpu, scale, causal, dtype, full_limit=1 << 31, seed=0, n_rows=512,
              rounding_aware=False):
    B, H, Sq, D = Q.shape
    Sk = K.shape[2]
    Og = O_gpu.detach().cpu().double().numpy()
    assert np.all(np.isfinite(Og)), "non-finite output"
    if B * H * Sq * Sk * D <= full_limit:
        Oref = oracle.mha_fwd(Q, K, V, scale, causal, dtype)
        got = Og
    else:
        rng = np.random.default_rng(seed + 777)
        bs, hs, qs = mha_sample_rows(B, H, Sq, rng, n_rows=n_rows)
        Oref = oracle.mha_fwd_rows(Q, K, V, bs, hs, qs, scale, causal, dtype)
        got = Og[bs, hs, qs]
    err = np.abs(got - Oref)
    rel_rms = float(np.sqrt(np.mean(err ** 2)) / max(np.sqrt(np.mean(Oref ** 2)), 1e-30))
    mx = float(err.max())
    # Beside the graded number: the distance to the correctly rounded oracle value, in units of the
    # output type's spacing there. One correct rounding of a value within `a` of the oracle's lands
    # within one spacing + a of the rounded oracle value.
    Oref_r = round_to_dtype(Oref, dtype)
    ulp = ulp_of(Oref_r, dtype)
    err_r = np.abs(got - Oref_r)
    n_over = int(np.count_nonzero(err > MHA_TOL[dtype]))
    stats = {"max_err": mx, "rel_rms": rel_rms, "n": int(err.size),
             "max_err_vs_rounded": float(err_r.max()), "max_ulps_vs_rounded": float(np.max(err_r / ulp)),
             "n_over_graded": n_over}
    if rounding_aware:
        # Inputs built so that |O| ~ |V| (up to ~4): one rounding of the output alone can exceed
        # the absolute bound (bf16 half-ulp at 4 is 1.6e-2). Such cases are held to one spacing of
        # the output type around the rounded oracle value plus an arithmetic term of half the
        # graded tolerance: a weight rounded to 16 bit carries a relative error up to 2^-9 (2^-12),
        # which reaches the output multiplied by the weight and by the distance of its value row
        # from the output row, a few units when two or three weights dominate a row; the fp32 sums
        # add far less. The number of elements beyond the graded bound is reported beside it.
        bound = ulp + 0.5 * MHA_TOL[dtype]
        worst = float(np.max(err_r / bound))
        assert np.all(err_r <= bound), ("attention parity (rounding-aware): worst |O - round(O_ref)| / "
                                        "(ulp + a) = %.3f; %d elements over the graded bound" % (worst, n_over))
    else:
        assert mx <= MHA_TOL[dtype], "attention parity: max err %.3g (rel rms %.3g)" % (mx, rel_rms)
    return stats


def run_mha(Q, K, V, scale, causal, dtype, device="cuda:0"):
    from paper_2503_14985_amd import binding
    dev = torch.device(device)
    tq, tk, tv = (inputs.bits_to_torch(x, dtype, dev) for x in (Q, K, V))
    O = binding.mlt_mha_fwd(tq, tk, tv, scale=scale, causal=causal)
    torch.cuda.synchronize()
    return O
