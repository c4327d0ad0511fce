"""CPU oracle (fp64, plain definitions) for the GEMM and attention-forward kernels.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the bench's cpu_baseline leg.
The GPU library never imports or links this package, and this package never touches the GPU
library. The arithmetic lives in ``oracle.c`` (GEMM: Section 2 / Listing 1 of arXiv 2503.14985;
attention: Section 2.5, Algorithm 1); this file only compiles it with gcc and marshals numpy
arrays of raw 16-bit patterns (``uint16``) through ctypes.

Paged attention for decoding (Section 3.2) is ``paged_attn_decode``.

dtype codes: 0 = bf16, 1 = fp16.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

BF16 = 0
FP16 = 1


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile oracle.c into liboracle.so with gcc (OpenMP for the outer-loop split)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        tmp = out + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, src, "-lm"])
        os.replace(tmp, out)
    return out


def _bind(path: str):
    lib = ctypes.CDLL(path)
    i64, p, dbl, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_double, ctypes.c_int
    lib.oracle_bf16_to_f64.restype = dbl
    lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_f16_to_f64.restype = dbl
    lib.oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
    lib.oracle_round_to_dtype.restype = dbl
    lib.oracle_round_to_dtype.argtypes = [dbl, i32]
    lib.oracle_num_threads.restype = i32
    lib.oracle_widen_array.restype = None
    lib.oracle_widen_array.argtypes = [p, i64, p, i32]
    lib.oracle_gemm.restype = i32
    lib.oracle_gemm.argtypes = [i64, i64, i64, p, i64, p, i64, i32, p, p, i32, i32]
    lib.oracle_gemm_sampled.restype = i32
    lib.oracle_gemm_sampled.argtypes = [i64, i64, i64, p, i64, p, i64, i32, i64, p, p, p, p,
                                        i32, i32]
    lib.oracle_gemm_epilogue.restype = i32
    lib.oracle_gemm_epilogue.argtypes = [i64, i64, p, i64, p, p, i32, i32]
    lib.oracle_mha_fwd.restype = i32
    lib.oracle_mha_fwd.argtypes = [i64, i64, i64, i64, i64, p, p, p, p, dbl, i32, i32, i32]
    lib.oracle_mha_fwd_rows.restype = i32
    lib.oracle_mha_fwd_rows.argtypes = [i64, i64, i64, i64, i64, p, p, p, i64, p, p, p, p, p,
                                        dbl, i32, i32, i32]
    lib.oracle_paged_attn_decode.restype = i32
    lib.oracle_paged_attn_decode.argtypes = [i64, i64, i64, i64, i64, i64, p, p, p, p, p, p, p,
                                             dbl, i32, i32]
    return lib


_lib = None
_override = None


def use_library(path):
    """Point the module at another build of oracle.c (tests that plant a mistake in a copy of
    the source use this); ``None`` restores the committed oracle."""
    global _override
    _override = _bind(path) if path is not None else None


def _load():
    global _lib
    if _override is not None:
        return _override
    if _lib is None:
        _lib = _bind(build())
    return _lib


def _u16(x: np.ndarray) -> np.ndarray:
    if x.dtype != np.uint16:
        raise TypeError("oracle inputs are raw 16-bit patterns (numpy uint16), got %s" % x.dtype)
    return x


def _ptr(x: np.ndarray):
    return x.ctypes.data_as(ctypes.c_void_p)


def _ld(x: np.ndarray) -> int:
    """Row stride in elements of a 2-D array whose rows are contiguous."""
    if x.shape[0] <= 1 or x.shape[1] == 0:
        return max(x.shape[1], 1)
    if x.strides[1] != 2:
        raise ValueError("rows must be contiguous")
    return x.strides[0] // 2


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Widen every 16-bit pattern exactly to float64 (element by element through oracle.c)."""
    flat = np.ascontiguousarray(_u16(bits)).ravel()
    out = np.empty(flat.shape, dtype=np.float64)
    _load().oracle_widen_array(_ptr(flat), flat.shape[0], _ptr(out), dtype)
    return out.reshape(bits.shape)


def scalar_to_f64(bits: int, dtype: int) -> float:
    lib = _load()
    fn = lib.oracle_bf16_to_f64 if dtype == BF16 else lib.oracle_f16_to_f64
    return float(fn(int(bits)))


def round_to_dtype(x: float, dtype: int) -> float:
    return float(_load().oracle_round_to_dtype(float(x), dtype))


def gemm(A: np.ndarray, B: np.ndarray, dtype: int, transB: bool = False, nthreads: int = 0):
    """Return (C_ref, T): C_ref = A*B and T = |A|*|B|, both float64 [M, N].

    A is [M, K] uint16. B is [K, N] uint16 (transB=False) or [N, K] uint16 (transB=True).
    Row strides are taken from the arrays, so padded leading dimensions work.
    """
    _u16(A), _u16(B)
    M, K = A.shape
    if transB:
        N, Kb = B.shape
    else:
        Kb, N = B.shape
    if K != Kb:
        raise ValueError("inner dimensions differ")
    lda, ldb = _ld(A), _ld(B)
    C = np.empty((M, N), dtype=np.float64)
    T = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm(M, N, K, _ptr(A), lda, _ptr(B), ldb, int(transB), _ptr(C), _ptr(T),
                             dtype, nthreads)
    if rc != 0:
        raise RuntimeError("oracle_gemm failed: %d" % rc)
    return C, T


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def gemm_bias_act(A, B, bias, act: int, dtype: int, transB: bool = False, nthreads: int = 0):
    """(Y_ref, T) for the fused GEMM Y = act(A*B + bias): the exact product from `gemm`, then the
    epilogue in fp64. bias is a uint16 [N] array in `dtype` or None; T = |A||B| + |bias|."""
    C, T = gemm(A, B, dtype, transB=transB, nthreads=nthreads)
    M, N = C.shape
    if bias is not None:
        _u16(bias)
        if bias.shape != (N,):
            raise ValueError("bias must have N elements")
        bias = np.ascontiguousarray(bias)
    rc = _load().oracle_gemm_epilogue(M, N, _ptr(C), N, _ptr(T), _ptr(bias) if bias is not None else None,
                                      int(act), dtype)
    if rc != 0:
        raise RuntimeError("oracle_gemm_epilogue failed: %d" % rc)
    return C, T


def gemm_sampled(A, B, rows, cols, dtype: int, transB: bool = False, nthreads: int = 0):
    """(C_ref, T) at the positions (rows[s], cols[s]) only; float64 [nsamples]."""
    _u16(A), _u16(B)
    M, K = A.shape
    N = B.shape[0] if transB else B.shape[1]
    lda, ldb = _ld(A), _ld(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    n = rows.shape[0]
    C = np.empty(n, dtype=np.float64)
    T = np.empty(n, dtype=np.float64)
    rc = _load().oracle_gemm_sampled(M, N, K, _ptr(A), lda, _ptr(B), ldb, int(transB), n,
                                     _ptr(rows), _ptr(cols), _ptr(C), _ptr(T), dtype, nthreads)
    if rc != 0:
        raise RuntimeError("oracle_gemm_sampled failed: %d" % rc)
    return C, T


def mha_fwd(Q, K, V, scale: float, causal: bool, dtype: int, nthreads: int = 0) -> np.ndarray:
    """O_ref float64 [B, H, Sq, D] for contiguous uint16 Q [B,H,Sq,D], K and V [B,H,Sk,D]."""
    Q, K, V = (np.ascontiguousarray(_u16(x)) for x in (Q, K, V))
    B, H, Sq, D = Q.shape
    Sk = K.shape[2]
    assert K.shape == (B, H, Sk, D) and V.shape == (B, H, Sk, D)
    O = np.empty((B, H, Sq, D), dtype=np.float64)
    rc = _load().oracle_mha_fwd(B, H, Sq, Sk, D, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), float(scale),
                                int(causal), dtype, nthreads)
    if rc != 0:
        raise RuntimeError("oracle_mha_fwd failed: %d" % rc)
    return O


def mha_fwd_rows(Q, K, V, bs, hs, qs, scale: float, causal: bool, dtype: int,
                 want_weights: bool = False, nthreads: int = 0):
    """O_ref float64 [nrows, D] for the rows (bs[r], hs[r], qs[r]); with want_weights also the
    softmax weights [nrows, Sk] (zeros at masked keys)."""
    Q, K, V = (np.ascontiguousarray(_u16(x)) for x in (Q, K, V))
    B, H, Sq, D = Q.shape
    Sk = K.shape[2]
    assert K.shape == (B, H, Sk, D) and V.shape == (B, H, Sk, D)
    bs, hs, qs = (np.ascontiguousarray(x, dtype=np.int64) for x in (bs, hs, qs))
    n = bs.shape[0]
    O = np.empty((n, D), dtype=np.float64)
    W = np.empty((n, Sk), dtype=np.float64) if want_weights else None
    rc = _load().oracle_mha_fwd_rows(B, H, Sq, Sk, D, _ptr(Q), _ptr(K), _ptr(V), n, _ptr(bs),
                                     _ptr(hs), _ptr(qs), _ptr(O), _ptr(W) if want_weights else None,
                                     float(scale), int(causal), dtype, nthreads)
    if rc != 0:
        raise RuntimeError("oracle_mha_fwd_rows failed: %d" % rc)
    return (O, W) if want_weights else O


def paged_attn_decode(Q, Kc, Vc, block_table, seq_lens, scale: float, dtype: int,
                      want_weights: bool = False, nthreads: int = 0):
    """O_ref float64 [B, H, D] of one query per (sequence, head) over a paged cache.

    Q [B,H,D] uint16; Kc, Vc [num_blocks, H, block_size, D] uint16; block_table [B, max_blocks]
    int32; seq_lens [B] int32. With want_weights also the softmax weights
    [B, H, max_blocks*block_size] (zeros beyond seq_len)."""
    Q, Kc, Vc = (np.ascontiguousarray(_u16(x)) for x in (Q, Kc, Vc))
    B, H, D = Q.shape
    nb, Hc, bs, Dc = Kc.shape
    assert (Hc, Dc) == (H, D) and Vc.shape == Kc.shape
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    assert block_table.shape[0] == B and seq_lens.shape == (B,)
    mb = block_table.shape[1]
    O = np.empty((B, H, D), dtype=np.float64)
    W = np.empty((B, H, mb * bs), dtype=np.float64) if want_weights else None
    rc = _load().oracle_paged_attn_decode(B, H, D, bs, mb, nb, _ptr(Q), _ptr(Kc), _ptr(Vc),
                                          _ptr(block_table), _ptr(seq_lens), _ptr(O),
                                          _ptr(W) if want_weights else None, float(scale), dtype,
                                          nthreads)
    if rc != 0:
        raise RuntimeError("oracle_paged_attn_decode failed: %d" % rc)
    return (O, W) if want_weights else O
