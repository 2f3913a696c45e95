"""ctypes binding of include/peak_gemm.h: same names, argument marshalling only.

Device buffers are passed as integer addresses (``tensor.data_ptr()``) and the
stream as ``torch.cuda.current_stream().cuda_stream``; PyTorch is used by the
callers for device memory and streams and for nothing else.
"""
from __future__ import annotations

import ctypes
import os

PEAK_DT_F32, PEAK_DT_F16, PEAK_DT_BF16 = 0, 1, 2
(PEAK_OK, PEAK_ERR_INVALID_ARG, PEAK_ERR_UNSUPPORTED, PEAK_ERR_WORKSPACE,
 PEAK_ERR_HIP, PEAK_ERR_ALLOC) = range(6)

PEAK_BIAS_NONE, PEAK_BIAS_PER_COLUMN, PEAK_BIAS_PER_ROW = 0, 1, 2
PEAK_ACT_NONE, PEAK_ACT_RELU, PEAK_ACT_GELU_TANH = 0, 1, 2
PEAK_GEMM_C_F32 = 0x10000
PEAK_GEMM_STREAMK_ON, PEAK_GEMM_STREAMK_OFF = 0x20000, 0x40000

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class PeakGemmDesc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64),
                ("transA", ctypes.c_int32), ("transB", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class PeakGemmEpilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("bias_kind", ctypes.c_int32), ("act", ctypes.c_int32)]


class PeakError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s: %s (status %d)" % (what, peak_status_string(status), status))
        self.status = status


def lib_path() -> str:
    """Path of the HIP library; PEAK_GEMM_LIB overrides it (to try another build)."""
    return os.environ.get("PEAK_GEMM_LIB") or os.path.join(_HERE, "libpeak_gemm.so")


def load_library():
    """Loads the HIP library.  Raises if it has not been built: there is no
    other implementation to fall back to."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError("libpeak_gemm.so is not built: run `python -m paper_2512_19018_amd.build` "
                              "(or __graft_entry__.build()) first")
        lib = ctypes.CDLL(path)
        P = ctypes.c_void_p
        lib.peak_gemm_create.restype = ctypes.c_int
        lib.peak_gemm_create.argtypes = [P, ctypes.POINTER(P)]
        lib.peak_gemm_workspace_bytes.restype = ctypes.c_size_t
        lib.peak_gemm_workspace_bytes.argtypes = [P]
        lib.peak_gemm_run.restype = ctypes.c_int
        lib.peak_gemm_run.argtypes = [P, ctypes.c_float, P, P, ctypes.c_float, P, P, ctypes.c_size_t, P]
        lib.peak_gemm_run_fused.restype = ctypes.c_int
        lib.peak_gemm_run_fused.argtypes = [P, ctypes.c_float, P, P, ctypes.c_float, P, P, P, ctypes.c_size_t, P]
        lib.peak_gemm_run_static.restype = ctypes.c_int
        lib.peak_gemm_run_static.argtypes = [P, ctypes.c_float, P, P, ctypes.c_float, P, P]
        lib.peak_gemm_destroy.restype = ctypes.c_int
        lib.peak_gemm_destroy.argtypes = [P]
        lib.peak_status_string.restype = ctypes.c_char_p
        lib.peak_status_string.argtypes = [ctypes.c_int]
        lib.peak_gemm_plan_info.restype = ctypes.c_int
        lib.peak_gemm_plan_info.argtypes = [P, ctypes.c_char_p, ctypes.c_size_t]
        lib.peak_gemm_variant_count.restype = ctypes.c_int
        lib.peak_gemm_variant_count.argtypes = []
        lib.peak_gemm_variant_name.restype = ctypes.c_char_p
        lib.peak_gemm_variant_name.argtypes = [ctypes.c_int]
        lib.peak_gemm_load_tuning.restype = ctypes.c_int
        lib.peak_gemm_load_tuning.argtypes = [ctypes.c_char_p]
        lib.peak_calib_mfma.restype = ctypes.c_int
        lib.peak_calib_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, P, P, ctypes.POINTER(ctypes.c_double)]
        lib.peak_calib_read.restype = ctypes.c_int
        lib.peak_calib_read.argtypes = [P, ctypes.c_size_t, P, P]
        lib.peak_calib_lds_load.restype = ctypes.c_int
        lib.peak_calib_lds_load.argtypes = [P, ctypes.c_size_t, ctypes.c_int32, P, P, ctypes.POINTER(ctypes.c_double),
                                            ctypes.POINTER(ctypes.c_int32)]
        _LIB = lib
    return _LIB


def peak_status_string(status: int) -> str:
    return load_library().peak_status_string(int(status)).decode()


def peak_gemm_variant_count() -> int:
    return load_library().peak_gemm_variant_count()


def peak_gemm_variant_name(i: int):
    s = load_library().peak_gemm_variant_name(int(i))
    return s.decode() if s is not None else None


def peak_gemm_load_tuning(path) -> int:
    """Load (or, with None, clear) the selector table; returns the number of entries, -1 on error."""
    return load_library().peak_gemm_load_tuning(None if path is None else os.fsencode(path))


def force_flags(variant: int | None = None, split: int | None = None, c_f32: bool = False,
                streamk: bool | None = None) -> int:
    """Descriptor flags that force a variant id and/or a K split, ask for an fp32 C, and
    switch hybrid stream-K on or off (None: the cost model decides)."""
    f = PEAK_GEMM_C_F32 if c_f32 else 0
    if streamk is not None:
        f |= PEAK_GEMM_STREAMK_ON if streamk else PEAK_GEMM_STREAMK_OFF
    if variant is not None:
        f |= (variant + 1) & 0xFF
    if split is not None:
        f |= (split & 0xFF) << 8
    return f


def peak_gemm_create(desc: PeakGemmDesc):
    """Returns (status, plan handle or None)."""
    h = ctypes.c_void_p()
    st = load_library().peak_gemm_create(ctypes.addressof(desc), ctypes.byref(h))
    return st, (h if st == PEAK_OK else None)


def peak_gemm_workspace_bytes(plan) -> int:
    return int(load_library().peak_gemm_workspace_bytes(plan))


def peak_gemm_run(plan, alpha: float, A: int, B: int, beta: float, C: int,
                  workspace: int = 0, workspace_bytes: int = 0, stream: int = 0) -> int:
    """A, B, C, workspace: device addresses (0 = NULL).  stream: hipStream_t as int."""
    return load_library().peak_gemm_run(plan, float(alpha), A or None, B or None, float(beta), C or None,
                                        workspace or None, int(workspace_bytes), stream or None)


def peak_gemm_run_fused(plan, alpha: float, A: int, B: int, beta: float, C: int, epilogue,
                        workspace: int = 0, workspace_bytes: int = 0, stream: int = 0) -> int:
    """As peak_gemm_run, with a PeakGemmEpilogue (or None) describing the fused output step."""
    ep = ctypes.addressof(epilogue) if epilogue is not None else None     # host struct, read during the call
    return load_library().peak_gemm_run_fused(plan, float(alpha), A or None, B or None, float(beta), C or None, ep,
                                              workspace or None, int(workspace_bytes), stream or None)


PEAK_GEMM_STATIC_WORKSPACE_BYTES = 32 << 20


def peak_gemm_run_static(plan, alpha: float, A: int, B: int, beta: float, C: int, stream: int = 0) -> int:
    """peak_gemm_run without a workspace argument: the partials go to the library's own fixed device array."""
    return load_library().peak_gemm_run_static(plan, float(alpha), A or None, B or None, float(beta), C or None,
                                               stream or None)


def peak_calib_mfma(dtype: int, random_operands: bool, iters: int, out_dev: int, stream: int = 0):
    """include/peak_calib.h: enqueues the MFMA-only loop; returns (status, flops of one launch)."""
    flops = ctypes.c_double(0.0)
    st = load_library().peak_calib_mfma(int(dtype), 1 if random_operands else 0, int(iters), out_dev or None,
                                        stream or None, ctypes.byref(flops))
    return st, flops.value


def peak_calib_lds_load(src_dev: int, nbytes: int, iters: int, out_dev: int, stream: int = 0):
    """include/peak_calib.h: enqueues the direct-to-LDS load loop; returns (status, bytes per workgroup, workgroups)."""
    b, n = ctypes.c_double(0.0), ctypes.c_int32(0)
    st = load_library().peak_calib_lds_load(src_dev or None, int(nbytes), int(iters), out_dev or None, stream or None,
                                            ctypes.byref(b), ctypes.byref(n))
    return st, b.value, n.value


def peak_calib_read(src_dev: int, nbytes: int, out_dev: int, stream: int = 0) -> int:
    """include/peak_calib.h: enqueues the read-only stream over [src_dev, src_dev + nbytes)."""
    return load_library().peak_calib_read(src_dev or None, int(nbytes), out_dev or None, stream or None)


def peak_gemm_destroy(plan) -> int:
    return load_library().peak_gemm_destroy(plan)


def peak_gemm_plan_info(plan) -> str:
    buf = ctypes.create_string_buffer(512)
    load_library().peak_gemm_plan_info(plan, buf, 512)
    return buf.value.decode()


class Plan:
    """Small RAII holder around a plan handle (create on init, destroy on close)."""

    def __init__(self, M, N, K, dtype, transA=0, transB=0, lda=None, ldb=None, ldc=None, flags=0):
        lda = lda if lda is not None else (M if transA else K)
        ldb = ldb if ldb is not None else (K if transB else N)
        ldc = ldc if ldc is not None else N
        self.desc = PeakGemmDesc(M, N, K, max(lda, 1), max(ldb, 1), max(ldc, 1), transA, transB, dtype, flags)
        st, h = peak_gemm_create(self.desc)
        if st != PEAK_OK:
            raise PeakError(st, "peak_gemm_create")
        self.handle = h
        self.workspace_bytes = peak_gemm_workspace_bytes(h)

    def info(self) -> str:
        return peak_gemm_plan_info(self.handle)

    def run(self, alpha, A, B, beta, C, workspace=0, workspace_bytes=0, stream=0):
        st = peak_gemm_run(self.handle, alpha, A, B, beta, C, workspace, workspace_bytes, stream)
        if st != PEAK_OK:
            raise PeakError(st, "peak_gemm_run")

    def run_fused(self, alpha, A, B, beta, C, bias_kind=PEAK_BIAS_NONE, bias=0, act=PEAK_ACT_NONE,
                  workspace=0, workspace_bytes=0, stream=0):
        ep = PeakGemmEpilogue(bias or None, bias_kind, act)
        st = peak_gemm_run_fused(self.handle, alpha, A, B, beta, C, ep, workspace, workspace_bytes, stream)
        if st != PEAK_OK:
            raise PeakError(st, "peak_gemm_run_fused")

    def close(self):
        if self.handle is not None:
            peak_gemm_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
