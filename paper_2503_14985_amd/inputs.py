"""Seeded synthetic inputs shared by the GPU path's tests/bench and by the oracle's callers.

This module holds none of the method's arithmetic: it draws fp32 values from numpy's
counter-seeded generator, rounds them to bf16 / fp16 with the library conversion of torch (CPU,
round-to-nearest-even) and returns the raw 16-bit patterns as ``uint16`` arrays. The same bytes
are handed to the GPU library and to the oracle, so no random-number code is shared.

The workloads are shape families only (GEMM sizes taken from LLM layer shapes; attention with a
fixed token budget, Section 4 of arXiv 2503.14985), so seeded random tensors are the workload.
"""
from __future__ import annotations

import numpy as np
import torch

BF16 = 0
FP16 = 1

_TORCH_DTYPE = {BF16: torch.bfloat16, FP16: torch.float16}
DTYPE_NAME = {BF16: "bf16", FP16: "fp16"}


def torch_dtype(dtype: int) -> torch.dtype:
    return _TORCH_DTYPE[dtype]


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round an fp32/fp64 array to the 16-bit format (RNE) and return the bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(_TORCH_DTYPE[dtype])
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_torch(bits: np.ndarray, dtype: int, device=None) -> torch.Tensor:
    """Reinterpret uint16 patterns as a torch tensor of the 16-bit dtype (optionally on a device)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(_TORCH_DTYPE[dtype])
    return t.to(device) if device is not None else t


def torch_to_bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a (possibly device) bf16/fp16 tensor, as a host uint16 array."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def _draw(rng: np.random.Generator, shape, dist: str, std: float) -> np.ndarray:
    if dist == "uniform":        # i.i.d. U[-1, 1]
        return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    if dist == "normal":         # i.i.d. N(0, std^2)
        return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std))
    raise ValueError(dist)


def gemm_inputs(M: int, N: int, K: int, dtype: int, seed: int, dist: str = "normal",
                std: float = 1.0, transB: bool = False, lda: int | None = None,
                ldb: int | None = None):
    """A [M, K] and B ([K, N], or [N, K] when transB) as uint16 patterns.

    With lda/ldb larger than the row length the returned arrays are views into padded buffers
    whose padding holds a NaN pattern, so a kernel that reads past a row is caught.
    """
    rng = np.random.default_rng(seed)
    a = to_bits(_draw(rng, (M, K), dist, std), dtype)
    bshape = (N, K) if transB else (K, N)
    b = to_bits(_draw(rng, bshape, dist, std), dtype)

    def pad(x, ld):
        if ld is None or ld == x.shape[1]:
            return x
        buf = np.full((x.shape[0], ld), 0x7FC1 if dtype == BF16 else 0x7E01, dtype=np.uint16)
        buf[:, : x.shape[1]] = x
        return buf[:, : x.shape[1]]

    return pad(a, lda), pad(b, ldb)


def bias_input(N: int, dtype: int, seed: int, std: float = 1.0) -> np.ndarray:
    """A bias vector of N values ~ N(0, std^2) as uint16 patterns (for the fused GEMM epilogue)."""
    rng = np.random.default_rng(seed + 7919)
    return to_bits(_draw(rng, (N,), "normal", std), dtype)


def mha_inputs(B: int, H: int, Sq: int, Sk: int, D: int, dtype: int, seed: int,
               q_gain: float = 1.0):
    """Q [B,H,Sq,D], K and V [B,H,Sk,D], i.i.d. N(0,1) (Q multiplied by q_gain), uint16 patterns."""
    rng = np.random.default_rng(seed)
    q = to_bits(_draw(rng, (B, H, Sq, D), "normal", q_gain), dtype)
    k = to_bits(_draw(rng, (B, H, Sk, D), "normal", 1.0), dtype)
    v = to_bits(_draw(rng, (B, H, Sk, D), "normal", 1.0), dtype)
    return q, k, v


def paged_inputs(B: int, H: int, D: int, block_size: int, seq_lens, dtype: int, seed: int,
                 extra_blocks: int = 3, shuffle: bool = True, poison: bool = False):
    """A paged KV cache for decoding: Q [B,H,D]; Kc, Vc [num_blocks, H, block_size, D]; block_table
    [B, max_blocks] int32; seq_lens [B] int32; plus the logical (dense) keys and values as lists of
    [H, len_b, D] arrays, from which the cache was filled. Values i.i.d. N(0,1). Physical blocks
    are handed out in a random order when `shuffle`; `extra_blocks` blocks stay unused. With
    `poison`, everything a correct reader never touches (slots past seq_len, unused blocks, table
    entries past the last block) holds NaN patterns / an out-of-range block number."""
    rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    assert seq_lens.shape == (B,) and seq_lens.min() >= 1
    nblk = (seq_lens.astype(np.int64) + block_size - 1) // block_size
    max_blocks = int(nblk.max())
    num_blocks = int(nblk.sum()) + extra_blocks
    q = to_bits(_draw(rng, (B, H, D), "normal", 1.0), dtype)
    fill = 0x7FC1 if dtype == BF16 else 0x7E01            # a NaN in either format
    kc = np.full((num_blocks, H, block_size, D), fill if poison else 0, dtype=np.uint16)
    vc = np.full((num_blocks, H, block_size, D), fill if poison else 0, dtype=np.uint16)
    table = np.full((B, max_blocks), num_blocks + 7 if poison else 0, dtype=np.int32)
    order = rng.permutation(num_blocks) if shuffle else np.arange(num_blocks)
    nxt = 0
    k_dense, v_dense = [], []
    for b in range(B):
        n = int(seq_lens[b])
        k = to_bits(_draw(rng, (H, n, D), "normal", 1.0), dtype)
        v = to_bits(_draw(rng, (H, n, D), "normal", 1.0), dtype)
        k_dense.append(k)
        v_dense.append(v)
        for i in range(int(nblk[b])):
            pb = int(order[nxt]); nxt += 1
            table[b, i] = pb
            lo, hi = i * block_size, min((i + 1) * block_size, n)
            kc[pb, :, : hi - lo, :] = k[:, lo:hi, :]
            vc[pb, :, : hi - lo, :] = v[:, lo:hi, :]
    return q, kc, vc, table, seq_lens, k_dense, v_dense
