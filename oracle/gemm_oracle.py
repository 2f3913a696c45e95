"""ctypes front end of the CPU oracle (oracle_gemm.c) and the error measure.

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the bench's CPU-baseline
leg call this; the GPU library never does, and this module imports nothing of
the GPU library.

``gemm`` returns the fp64 reference of C = alpha*op(A)*op(B) + beta*C_in for
stored arrays (Section 2.2 of the paper: C = A x B, row-major, one dot product
per output element; widened to the BLAS form).  ``rel_frobenius`` is the
acceptance measure: ||C_gpu - ref||_F / ||ref||_F.  ``bias_act`` is the fused
output step act(ref + bias) (Section 1.2: a MatMul open to fusion-style
modifications), in fp64, on a finished reference.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_gemm.so")
_lib = None

F32, F16, BF16 = 0, 1, 2
BIAS_NONE, BIAS_PER_COLUMN, BIAS_PER_ROW = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_GELU_TANH = 0, 1, 2


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_gemm.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_double, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_double, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        lib.oracle_gemm_c.restype = ctypes.c_int
        lib.oracle_gemm_c.argtypes = [ctypes.c_int] + lib.oracle_gemm.argtypes
        lib.oracle_bias_act.restype = ctypes.c_int
        lib.oracle_bias_act.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_decode_f16.restype = ctypes.c_double
        lib.oracle_decode_f16.argtypes = [ctypes.c_uint16]
        lib.oracle_decode_bf16.restype = ctypes.c_double
        lib.oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        _lib = lib
    return _lib


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:
        return max(1, os.cpu_count() or 1)


def decode_f16(bits: int) -> float:
    return _load().oracle_decode_f16(int(bits))


def decode_bf16(bits: int) -> float:
    return _load().oracle_decode_bf16(int(bits))


def _check_storage(x: np.ndarray, dtype: int, name: str):
    want = np.float32 if dtype == F32 else np.uint16
    if x.dtype != want or x.ndim != 2 or not x.flags.c_contiguous:
        raise ValueError("%s must be a C-contiguous 2-D %s array" % (name, np.dtype(want).name))


def gemm(dtype: int, transA: int, transB: int, M: int, N: int, K: int,
         alpha: float, A: np.ndarray, B: np.ndarray, beta: float = 0.0,
         Cin: np.ndarray | None = None, rows=None, order: int = -1,
         threads: int | None = None, cdtype: int | None = None) -> np.ndarray:
    """fp64 reference.  A, B, Cin are the arrays *as stored* (2-D, their row
    length is the leading dimension).  ``rows``: optional list of logical row
    indices of C; the result then has one row per entry.  ``cdtype``: storage
    type of Cin when it differs from that of A and B."""
    lib = _load()
    _check_storage(A, dtype, "A")
    _check_storage(B, dtype, "B")
    lda, ldb = A.shape[1], B.shape[1]
    ldc = 0
    cptr = None
    if Cin is not None:
        _check_storage(Cin, dtype if cdtype is None else cdtype, "Cin")
        ldc = Cin.shape[1]
        cptr = Cin.ctypes.data
    a_rows_needed = K if transA else M
    b_rows_needed = N if transB else K
    if A.shape[0] < a_rows_needed or B.shape[0] < b_rows_needed:
        raise ValueError("stored operand has too few rows")
    if Cin is not None and Cin.shape[0] < M:
        raise ValueError("C_in has too few rows")
    rptr, nrows = None, 0
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rptr, nrows = rows.ctypes.data, rows.size
    out_rows = nrows if rows is not None else M
    ref = np.empty((out_rows, N), dtype=np.float64)
    a32 = float(np.float32(alpha))
    b32 = float(np.float32(beta))
    rc = lib.oracle_gemm_c(dtype, dtype if cdtype is None else int(cdtype), int(transA), int(transB), M, N, K,
                         a32, A.ctypes.data, lda, B.ctypes.data, ldb,
                         b32, cptr, ldc, rptr, nrows,
                         ref.ctypes.data, order, threads or default_threads())
    if rc != 0:
        raise ValueError("oracle_gemm rejected its arguments")
    return ref


def bias_act(ref: np.ndarray, M: int, bias_kind: int = BIAS_NONE, bias: np.ndarray | None = None,
             act: int = ACT_NONE, rows=None) -> np.ndarray:
    """act(ref + bias) in fp64, in a new array.  ``ref`` is what ``gemm`` returned for
    an M-row problem (all rows, or the logical rows listed in ``rows``); ``bias`` holds
    fp32 values, one per column (BIAS_PER_COLUMN) or per logical row (BIAS_PER_ROW)."""
    lib = _load()
    out = np.array(ref, dtype=np.float64, order="C", copy=True)
    if out.ndim != 2:
        raise ValueError("ref must be 2-D")
    N = out.shape[1]
    bptr = None
    if bias_kind != BIAS_NONE:
        if bias is None or bias.dtype != np.float32 or bias.ndim != 1 or not bias.flags.c_contiguous:
            raise ValueError("bias must be a contiguous 1-D float32 array")
        if bias.size < (N if bias_kind == BIAS_PER_COLUMN else M):
            raise ValueError("bias is too short")
        bptr = bias.ctypes.data
    rptr, nrows = None, 0
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rptr, nrows = rows.ctypes.data, rows.size
    if out.shape[0] != (nrows if rows is not None else M):
        raise ValueError("ref has the wrong number of rows")
    rc = lib.oracle_bias_act(M, N, rptr, nrows, out.ctypes.data, int(bias_kind), bptr, int(act))
    if rc != 0:
        raise ValueError("oracle_bias_act rejected its arguments")
    return out


def rel_frobenius(c: np.ndarray, ref: np.ndarray) -> float:
    """||c - ref||_F / ||ref||_F in fp64.  A non-finite entry of c where ref is
    finite gives inf.  If ref is all zero, returns 0.0 only when c is too."""
    c = np.asarray(c, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if c.shape != ref.shape:
        raise ValueError("shape mismatch %s vs %s" % (c.shape, ref.shape))
    if c.size == 0:
        return 0.0
    if np.any(~np.isfinite(c) & np.isfinite(ref)):
        return float("inf")
    num = float(np.sqrt(np.sum((c - ref) ** 2)))
    den = float(np.sqrt(np.sum(ref ** 2)))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
