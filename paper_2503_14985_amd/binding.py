"""ctypes binding of libmlt.so: the same names as the C ABI in include/mlt.h, argument marshalling
only. Every step of both operations runs in the HIP kernels; there is no fallback: if the
library has not been built, importing this module raises.

Tensors are torch tensors on the GPU (bf16 or fp16); torch is used for device memory and the
current stream, nothing else.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmlt.so")

MLT_BF16, MLT_FP16 = 0, 1
MLT_OK, MLT_ERR_INVALID_ARG, MLT_ERR_UNSUPPORTED, MLT_ERR_LAUNCH, MLT_ERR_DEVICE = 0, -1, -2, -3, -4
MLT_ERR_SCRATCH = -5

# include/mlt.h (the operations) and include/mlt_diag.h (probes, timing hooks, kernel-choice overrides)
EXPORTS = ("mlt_gemm", "mlt_gemm_noalloc", "mlt_gemm_acc", "mlt_gemm_tiled", "mlt_gemm_bias_act", "mlt_mha_fwd",
           "mlt_paged_attn_decode", "mlt_status_string", "mlt_version")
DIAG_EXPORTS = ("mlt_probe_mfma", "mlt_probe_mfma16", "mlt_probe_hbm_read", "mlt_set_timing_events",
                "mlt_last_kernel", "mlt_query_tiling", "mlt_diag_force_variant",
                "mlt_diag_force_k_parts", "mlt_diag_force_key_split", "mlt_diag_set_persistent_grid")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmlt.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build_lib()'` "
        "from the repository root; there is no CPU fallback." % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)
_i64, _p, _i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
_lib.mlt_gemm.restype = _i32
_lib.mlt_gemm.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _p]
_lib.mlt_gemm_noalloc.restype = _i32
_lib.mlt_gemm_noalloc.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _p]
_lib.mlt_gemm_acc.restype = _i32
_lib.mlt_gemm_acc.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _p]
_lib.mlt_gemm_tiled.restype = _i32
_lib.mlt_gemm_tiled.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i64, _i32, _i32, _p]
_lib.mlt_gemm_bias_act.restype = _i32
_lib.mlt_gemm_bias_act.argtypes = [_i64, _i64, _i64, _p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _i32, _p]
_lib.mlt_mha_fwd.restype = _i32
_lib.mlt_mha_fwd.argtypes = [_i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, ctypes.c_float, _i32,
                             _i32, _p]
_lib.mlt_paged_attn_decode.restype = _i32
_lib.mlt_paged_attn_decode.argtypes = [_i64, _i64, _i64, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p,
                                       ctypes.c_float, _i32, _p]
_lib.mlt_probe_mfma.restype = _i32
_lib.mlt_probe_mfma.argtypes = [_i32, _p, _p, ctypes.POINTER(ctypes.c_double), _p]
_lib.mlt_probe_mfma16.restype = _i32
_lib.mlt_probe_mfma16.argtypes = [_i32, _p, _p, ctypes.POINTER(ctypes.c_double), _p]
_lib.mlt_probe_hbm_read.restype = _i32
_lib.mlt_probe_hbm_read.argtypes = [_p, _i64, _p, _p]
_lib.mlt_set_timing_events.restype = None
_lib.mlt_set_timing_events.argtypes = [_p, _p]
_lib.mlt_last_kernel.restype = ctypes.c_char_p
_lib.mlt_query_tiling.restype = _i32
_lib.mlt_query_tiling.argtypes = [_i32, ctypes.POINTER(_i64), _i32, ctypes.POINTER(ctypes.c_int32)]
_lib.mlt_diag_force_variant.restype = _i32
_lib.mlt_diag_force_variant.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
_lib.mlt_diag_force_k_parts.restype = _i32
_lib.mlt_diag_force_k_parts.argtypes = [_i32]
_lib.mlt_diag_force_key_split.restype = _i32
_lib.mlt_diag_force_key_split.argtypes = [_i32]
_lib.mlt_diag_set_persistent_grid.restype = _i32
_lib.mlt_diag_set_persistent_grid.argtypes = [_i32]
_lib.mlt_status_string.restype = ctypes.c_char_p
_lib.mlt_status_string.argtypes = [_i32]
_lib.mlt_version.restype = ctypes.c_char_p


class MltError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, mlt_status_string(status), status))


def raw():
    """The ctypes library object, for tests that pass raw pointers (error paths)."""
    return _lib


def mlt_status_string(status: int) -> str:
    return _lib.mlt_status_string(status).decode()


def mlt_version() -> str:
    return _lib.mlt_version().decode()


def mlt_last_kernel() -> str:
    return _lib.mlt_last_kernel().decode()


def mlt_diag_force_variant(gemm: str | None = None, mha: str | None = None) -> None:
    """Force a GEMM and/or attention kernel variant for the whole process (None: leave as is,
    "auto": the library's own choice)."""
    rc = _lib.mlt_diag_force_variant(None if gemm is None else gemm.encode(),
                                     None if mha is None else mha.encode())
    if rc != MLT_OK:
        raise MltError(rc, "mlt_diag_force_variant")


def mlt_diag_force_k_parts(parts: int) -> None:
    """0: the library's choice; 1: no K split across workgroups; 2 / 4 / 8: that many parts."""
    rc = _lib.mlt_diag_force_k_parts(int(parts))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_diag_force_k_parts")


def mlt_diag_force_key_split(ranges: int) -> None:
    """Paged decode: 0 = the library's choice; 1..64 = key ranges per (sequence, head)."""
    rc = _lib.mlt_diag_force_key_split(int(ranges))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_diag_force_key_split")


def mlt_diag_set_persistent_grid(workgroups: int) -> None:
    rc = _lib.mlt_diag_set_persistent_grid(int(workgroups))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_diag_set_persistent_grid")


def mlt_paged_attn_decode(Q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor,
                          block_table: torch.Tensor, seq_lens: torch.Tensor, scale: float,
                          O: torch.Tensor = None) -> torch.Tensor:
    """Q [B,H,D]; Kc, Vc [num_blocks,H,block_size,D]; block_table int32 [B,max_blocks]; seq_lens
    int32 [B]; returns O [B,H,D]. All on the GPU, contiguous."""
    B, H, D = Q.shape
    nb, Hc, bs, Dc = Kc.shape
    if (Hc, Dc) != (H, D) or Vc.shape != Kc.shape or Vc.dtype != Q.dtype or Kc.dtype != Q.dtype:
        raise ValueError("mlt_paged_attn_decode: cache shape/dtype does not match Q")
    if block_table.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise ValueError("mlt_paged_attn_decode: block_table and seq_lens must be int32")
    if block_table.shape[0] != B or tuple(seq_lens.shape) != (B,):
        raise ValueError("mlt_paged_attn_decode: block_table / seq_lens shape")
    for t in (Q, Kc, Vc, block_table, seq_lens):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("mlt_paged_attn_decode: tensors must be contiguous GPU tensors")
    if O is None:
        O = torch.empty_like(Q)
    rc = _lib.mlt_paged_attn_decode(B, H, D, bs, block_table.shape[1], nb, Q.data_ptr(),
                                    Kc.data_ptr(), Vc.data_ptr(), block_table.data_ptr(),
                                    seq_lens.data_ptr(), O.data_ptr(), float(scale),
                                    _dtype_code(Q), torch.cuda.current_stream(Q.device).cuda_stream)
    if rc != MLT_OK:
        raise MltError(rc, "mlt_paged_attn_decode")
    return O


def mlt_probe_mfma(iters: int, data: torch.Tensor, sink: torch.Tensor, mfma_size: int = 32) -> float:
    """Enqueue the register-only MFMA loop on the current stream; returns the flop it executes.
    `data`: at least 64 KiB of bf16 operand values on the GPU, `sink`: at least 4 bytes.
    mfma_size 32: 32x32x16 MFMAs (mlt_probe_mfma), 16: 16x16x32 (mlt_probe_mfma16)."""
    if not data.is_cuda or data.numel() * data.element_size() < 65536 or not data.is_contiguous():
        raise ValueError("mlt_probe_mfma: data must be a contiguous GPU tensor of at least 64 KiB")
    if mfma_size not in (16, 32):
        raise ValueError("mfma_size must be 16 or 32")
    fn = _lib.mlt_probe_mfma16 if mfma_size == 16 else _lib.mlt_probe_mfma
    flop = ctypes.c_double()
    rc = fn(int(iters), data.data_ptr(), sink.data_ptr(), ctypes.byref(flop),
            torch.cuda.current_stream(data.device).cuda_stream)
    if rc != MLT_OK:
        raise MltError(rc, "mlt_probe_mfma")
    return flop.value


def mlt_probe_mfma16(iters: int, data: torch.Tensor, sink: torch.Tensor) -> float:
    return mlt_probe_mfma(iters, data, sink, mfma_size=16)


def mlt_probe_hbm_read(data: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueue the read-only streaming kernel over `data` (contiguous GPU tensor, a multiple of 16
    bytes) on the current stream; returns the bytes it reads."""
    nbytes = data.numel() * data.element_size()
    if not data.is_cuda or not data.is_contiguous():
        raise ValueError("mlt_probe_hbm_read: data must be a contiguous GPU tensor")
    rc = _lib.mlt_probe_hbm_read(data.data_ptr(), nbytes, sink.data_ptr(),
                                 torch.cuda.current_stream(data.device).cuda_stream)
    if rc != MLT_OK:
        raise MltError(rc, "mlt_probe_hbm_read")
    return nbytes


def mlt_query_tiling(op: int, dims, dtype: int):
    d = (_i64 * 4)(*[int(x) for x in dims])
    out = (ctypes.c_int32 * 10)()
    rc = _lib.mlt_query_tiling(op, d, dtype, out)
    if rc != MLT_OK:
        raise MltError(rc, "mlt_query_tiling")
    return list(out)


def mlt_set_timing_events(start, stop) -> None:
    """start/stop: raw hipEvent_t handles as ints (or None)."""
    _lib.mlt_set_timing_events(start, stop)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MLT_BF16
    if t.dtype == torch.float16:
        return MLT_FP16
    raise TypeError("mlt works on bfloat16 / float16 tensors, got %s" % t.dtype)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _rows_contiguous(t: torch.Tensor, name: str) -> int:
    if t.dim() != 2:
        raise ValueError("%s must be 2-D" % name)
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError("%s must have contiguous rows" % name)
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)


def _gemm_operands(name: str, A, B, C, transB: bool, c_dtype=None):
    """Shapes, dtype code and leading dimensions of a GEMM call (C allocated when None): the
    marshalling every GEMM entry point shares."""
    if not (A.is_cuda and B.is_cuda and (C is None or C.is_cuda)):
        raise ValueError("%s needs GPU tensors" % name)
    dt = _dtype_code(A)
    if B.dtype != A.dtype:
        raise TypeError("A and B must share a dtype")
    M, K = A.shape
    N, Kb = (B.shape[0], B.shape[1]) if transB else (B.shape[1], B.shape[0])
    if K != Kb:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, Kb))
    c_dtype = A.dtype if c_dtype is None else c_dtype
    if C is None:
        C = torch.empty((M, N), dtype=c_dtype, device=A.device)
    elif C.dtype != c_dtype or tuple(C.shape) != (M, N):
        raise ValueError("C has the wrong dtype or shape")
    lda, ldb, ldc = _rows_contiguous(A, "A"), _rows_contiguous(B, "B"), _rows_contiguous(C, "C")
    return M, N, K, lda, ldb, ldc, dt, C


def mlt_gemm(A: torch.Tensor, B: torch.Tensor, C: torch.Tensor | None = None, transB: bool = False,
             stream=None) -> torch.Tensor:
    """C = A @ B (transB=False, B is [K, N]) or C = A @ B.T (transB=True, B is [N, K]).

    Row strides of A, B and C are passed through as lda/ldb/ldc, so row-sliced views work."""
    M, N, K, lda, ldb, ldc, dt, C = _gemm_operands("mlt_gemm", A, B, C, transB)
    with torch.cuda.device(A.device):
        rc = _lib.mlt_gemm(M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, int(transB),
                           C.data_ptr(), ldc, dt, _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_gemm")
    return C


def mlt_gemm_noalloc(A: torch.Tensor, B: torch.Tensor, C: torch.Tensor, transB: bool = False,
                     stream=None) -> torch.Tensor:
    """mlt_gemm through the entry point that allocates nothing: C must be given."""
    if C is None:
        raise ValueError("mlt_gemm_noalloc needs the C it writes (this wrapper allocates nothing)")
    M, N, K, lda, ldb, ldc, dt, C = _gemm_operands("mlt_gemm_noalloc", A, B, C, transB)
    with torch.cuda.device(A.device):
        rc = _lib.mlt_gemm_noalloc(M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, int(transB),
                                   C.data_ptr(), ldc, dt, _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_gemm_noalloc")
    return C


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
TILING_AUTO, TILING_HORIZONTAL, TILING_VERTICAL, TILING_SQUARE = 0, 1, 2, 3


def mlt_gemm_tiled(A: torch.Tensor, B: torch.Tensor, tiling: int, C: torch.Tensor | None = None,
                   transB: bool = False, stream=None) -> torch.Tensor:
    """mlt_gemm with the paper's tiling hint (TILING_AUTO / _HORIZONTAL / _VERTICAL / _SQUARE)."""
    M, N, K, lda, ldb, ldc, dt, C = _gemm_operands("mlt_gemm_tiled", A, B, C, transB)
    with torch.cuda.device(A.device):
        rc = _lib.mlt_gemm_tiled(M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, int(transB),
                                 C.data_ptr(), ldc, dt, int(tiling), _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_gemm_tiled")
    return C


def mlt_gemm_bias_act(A: torch.Tensor, B: torch.Tensor, bias: torch.Tensor | None = None,
                      act: int = ACT_NONE, C: torch.Tensor | None = None, transB: bool = False,
                      stream=None) -> torch.Tensor:
    """C = act(A @ B + bias) (or A @ B.T), bias a contiguous [N] tensor of the input dtype or None,
    act one of ACT_NONE / ACT_RELU / ACT_GELU."""
    M, N, K, lda, ldb, ldc, dt, C = _gemm_operands("mlt_gemm_bias_act", A, B, C, transB)
    if bias is not None and (not bias.is_cuda or bias.dtype != A.dtype or tuple(bias.shape) != (N,)
                             or not bias.is_contiguous()):
        raise ValueError("bias must be a contiguous GPU tensor of N elements of the input dtype")
    with torch.cuda.device(A.device):
        rc = _lib.mlt_gemm_bias_act(M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, int(transB),
                                    bias.data_ptr() if bias is not None else None, int(act),
                                    C.data_ptr(), ldc, dt, _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_gemm_bias_act")
    return C


def mlt_gemm_acc(A: torch.Tensor, B: torch.Tensor, C: torch.Tensor, transB: bool = False,
                 stream=None) -> torch.Tensor:
    """C += A @ B (or A @ B.T) with C an fp32 [M, N] tensor that is read and written."""
    if C is None:
        raise ValueError("mlt_gemm_acc needs the fp32 C it accumulates into")
    M, N, K, lda, ldb, ldc, dt, C = _gemm_operands("mlt_gemm_acc", A, B, C, transB, torch.float32)
    with torch.cuda.device(A.device):
        rc = _lib.mlt_gemm_acc(M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, int(transB),
                               C.data_ptr(), ldc, dt, _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_gemm_acc")
    return C


def mlt_mha_fwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, scale: float,
                causal: bool = False, O: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """O = softmax(scale * Q K^T [+ causal mask]) V for contiguous [B, H, S, D] tensors."""
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("mlt_mha_fwd needs GPU tensors")
    dt = _dtype_code(Q)
    if K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise TypeError("Q, K and V must share a dtype")
    if Q.dim() != 4 or K.dim() != 4 or V.shape != K.shape:
        raise ValueError("expected Q [B,H,Sq,D], K and V [B,H,Sk,D]")
    B, H, Sq, D = Q.shape
    Sk = K.shape[2]
    if K.shape != (B, H, Sk, D):
        raise ValueError("K shape does not match Q")
    if not (Q.is_contiguous() and K.is_contiguous() and V.is_contiguous()):
        raise ValueError("Q, K and V must be contiguous")
    if O is None:
        O = torch.empty_like(Q)
    elif O.dtype != Q.dtype or O.shape != Q.shape or not O.is_contiguous():
        raise ValueError("O has the wrong dtype, shape or layout")
    with torch.cuda.device(Q.device):
        rc = _lib.mlt_mha_fwd(B, H, Sq, Sk, D, Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                              O.data_ptr(), float(scale), int(causal), dt, _stream(stream))
    if rc != MLT_OK:
        raise MltError(rc, "mlt_mha_fwd")
    return O
