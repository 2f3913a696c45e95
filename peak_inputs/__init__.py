"""Seeded synthetic matrices for the GEMM workloads.

This module only makes inputs.  It holds none of the GEMM arithmetic and is the
one piece shared by the CPU oracle's tests and the HIP library's tests/bench:
both sides receive the very same host buffers, already rounded to the storage
dtype, so neither ever sees an unrounded value.

Generator: counter based, so any element can be produced on its own and the
result does not depend on chunking or threading.  With ``mix`` the splitmix64
output finaliser,

    base = mix(seed * GOLDEN + (stream + 1) * STREAM_MUL)
    x(e) = mix(base + (e + 1) * GOLDEN)                    (all mod 2**64)

where ``e`` is the row-major index of the element in the *logical* matrix
op(X) (rows x cols), whatever the storage layout.  Streams: 0 = A, 1 = B,
2 = C_in.

* uniform[-1, 1):  ((x >> 40) * 2**-24) * 2 - 1          (exact in fp32)
* normal(0, 1):    Box-Muller on u1 = ((x >> 40) + 1) * 2**-24 in (0, 1] and
                   u2 = ((x >> 16) & 0xFFFFFF) * 2**-24, evaluated in fp64,
                   then cast to fp32.

Values are scaled in fp32 and rounded once (round to nearest even) to the
storage dtype.  16-bit matrices are returned as ``uint16`` bit patterns.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

F32, F16, BF16 = 0, 1, 2          # same numbering as the C ABI's dtype enum
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}
DTYPE_SIZE = {F32: 4, F16: 2, BF16: 2}

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_STREAM_MUL = np.uint64(0xD1B54A32D192ED03)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def raw_bits(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """64-bit words x(e) for e in [start, start+count)."""
    with np.errstate(over="ignore"):
        base = _mix(np.array([np.uint64(seed) * _GOLDEN
                              + np.uint64(stream + 1) * _STREAM_MUL], dtype=np.uint64))[0]
        e = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(base + e * _GOLDEN)


def _uniform_from_bits(x: np.ndarray) -> np.ndarray:
    u = (x >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)
    return u * np.float32(2.0) - np.float32(1.0)


def _normal_from_bits(x: np.ndarray) -> np.ndarray:
    u1 = ((x >> np.uint64(40)).astype(np.float64) + 1.0) * 2.0 ** -24
    u2 = ((x >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * 2.0 ** -24
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return z.astype(np.float32)


def f32_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest even), returned as uint16 bit patterns."""
    b = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    r = np.where(nan, (b >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(v: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 values -> storage array (float32, or uint16 bit patterns)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    if dtype == F32:
        return v
    if dtype == F16:
        return v.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        return f32_to_bf16_bits(v)
    raise ValueError("unknown dtype %r" % (dtype,))


def to_f64(stored: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> float64 values (numpy's own decoders, used by tests)."""
    if dtype == F32:
        return stored.astype(np.float64)
    if dtype == F16:
        return stored.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(stored).astype(np.float64)
    raise ValueError("unknown dtype %r" % (dtype,))


def storage_np_dtype(dtype: int):
    return np.float32 if dtype == F32 else np.uint16


def logical_matrix(seed: int, stream: int, rows: int, cols: int, dist: str,
                   scale: float, dtype: int) -> np.ndarray:
    """rows x cols logical matrix, rounded to ``dtype``, C-contiguous."""
    n = rows * cols
    out = np.empty(n, dtype=storage_np_dtype(dtype))
    sc = np.float32(scale)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        x = raw_bits(seed, stream, s, c)
        if dist == "uniform":
            v = _uniform_from_bits(x)
        elif dist == "normal":
            v = _normal_from_bits(x)
        else:
            raise ValueError(dist)
        if scale != 1.0:
            v = v * sc
        out[s:s + c] = round_to_dtype(v, dtype)
    return out.reshape(rows, cols)


def store(logical: np.ndarray, trans: bool, ld: int | None = None, pad_value=None) -> np.ndarray:
    """Lay a logical op(X) matrix out as stored: transposed if ``trans``, with
    row stride ``ld`` (elements).  Padding beyond the row is ``pad_value``
    (default: a NaN pattern for the dtype) so that any read of it shows."""
    m = np.ascontiguousarray(logical.T if trans else logical)
    r, c = m.shape
    if ld is None or ld == c:
        return m
    if ld < c:
        raise ValueError("ld below the row length")
    if pad_value is None:
        pad_value = np.float32(np.nan) if m.dtype == np.float32 else np.uint16(0x7FC1)
    out = np.full((r, ld), pad_value, dtype=m.dtype)
    out[:, :c] = m
    return out


@dataclasses.dataclass(frozen=True)
class Workload:
    """One GEMM problem: C = alpha * op(A) * op(B) + beta * C_in."""
    name: str
    dtype: int
    M: int
    N: int
    K: int
    transA: int
    transB: int
    alpha: float
    beta: float
    dist: str          # "uniform" or "normal"
    scale: float       # multiplies every A and B entry before rounding
    seed: int
    note: str = ""

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K

    @property
    def esize(self) -> int:
        return DTYPE_SIZE[self.dtype]

    @property
    def min_bytes(self) -> float:
        """Algorithmic HBM bytes: each operand read once, C written once
        (and read once when beta != 0)."""
        e = self.esize
        c = self.M * self.N * e
        return (self.M * self.K + self.K * self.N) * e + c * (2 if self.beta != 0 else 1)

    def make(self, with_cin: bool | None = None):
        """Returns (A_stored, B_stored, C_in or None) with minimal leading dims."""
        a = logical_matrix(self.seed, 0, self.M, self.K, self.dist, self.scale, self.dtype)
        b = logical_matrix(self.seed, 1, self.K, self.N, self.dist, self.scale, self.dtype)
        need_c = (self.beta != 0) if with_cin is None else with_cin
        c = logical_matrix(self.seed, 2, self.M, self.N, self.dist, 1.0, self.dtype) if need_c else None
        return store(a, bool(self.transA)), store(b, bool(self.transB)), c

    def ld(self):
        lda = self.M if self.transA else self.K
        ldb = self.K if self.transB else self.N
        return lda, ldb, self.N


# The five graded configurations (C1..C5) plus the 4096^3 bf16 shape named in
# the target, and the square fp32/f16 shapes the paper itself measures
# (Section 4.3: n = 2048 and 4096, row-major, C = A x B).
WORKLOADS = {
    "C1": Workload("C1", F32, 256, 256, 256, 0, 0, 1.0, 0.0, "uniform", 1.0, 0,
                   "fp32 256^3 NN"),
    "C2": Workload("C2", F32, 4096, 4096, 4096, 0, 0, 1.0, 0.5, "uniform", 1.0, 1,
                   "fp32 4096^3 NN, beta=0.5"),
    "C3": Workload("C3", BF16, 8192, 8192, 8192, 0, 1, 1.0, 0.0, "normal", 1.0 / math.sqrt(8192.0), 2,
                   "bf16 8192^3 NT"),
    "C3b": Workload("C3b", BF16, 4096, 4096, 4096, 0, 1, 1.0, 0.0, "normal", 1.0 / math.sqrt(4096.0), 2,
                    "bf16 4096^3 NT"),
    "C4": Workload("C4", F16, 5000, 3000, 12288, 0, 0, 1.0, 0.0, "uniform", 1.0, 3,
                   "f16 5000x3000x12288 NN, ragged tiles"),
    "C5": Workload("C5", BF16, 16, 16384, 16384, 0, 1, 1.0, 0.0, "normal", 0.02, 4,
                   "bf16 skinny 16x16384x16384 NT (HBM bound)"),
    "P2k_f32": Workload("P2k_f32", F32, 2048, 2048, 2048, 0, 0, 1.0, 0.0, "uniform", 1.0, 5,
                        "paper shape fp32 2048^2 NN"),
    "P4k_f32": Workload("P4k_f32", F32, 4096, 4096, 4096, 0, 0, 1.0, 0.0, "uniform", 1.0, 6,
                        "paper shape fp32 4096^2 NN"),
    "P2k_f16": Workload("P2k_f16", F16, 2048, 2048, 2048, 0, 0, 1.0, 0.0, "uniform", 1.0, 7,
                        "paper shape f16 2048^2 NN"),
    "P4k_f16": Workload("P4k_f16", F16, 4096, 4096, 4096, 0, 0, 1.0, 0.0, "uniform", 1.0, 8,
                        "paper shape f16 4096^2 NN"),
    # 576 tiles of 256 x 256: two full rounds over 256 compute units and a quarter of a third (hybrid stream-K)
    "SK_bf16": Workload("SK_bf16", BF16, 8192, 4608, 8192, 0, 1, 1.0, 0.0, "normal", 1.0 / math.sqrt(8192.0), 11,
                        "bf16 8192x4608x8192 NT, 2.25 rounds of tiles"),
    # skinny products outside M <= 16 / 16 bits / B along K: the streaming path's other cases (HBM bound)
    "S32_bf16": Workload("S32_bf16", BF16, 32, 28672, 8192, 0, 1, 1.0, 0.0, "normal", 0.02, 12,
                         "bf16 skinny 32x28672x8192 NT (HBM bound)"),
    "S64_f16": Workload("S64_f16", F16, 64, 28672, 8192, 0, 1, 1.0, 0.0, "normal", 0.02, 13,
                        "f16 skinny 64x28672x8192 NT (HBM bound)"),
    "S16_f32": Workload("S16_f32", F32, 16, 16384, 16384, 0, 1, 1.0, 0.0, "normal", 0.02, 14,
                        "fp32 skinny 16x16384x16384 NT (HBM bound)"),
    "S16_bf16_kn": Workload("S16_bf16_kn", BF16, 16, 28672, 8192, 0, 0, 1.0, 0.0, "normal", 0.02, 15,
                            "bf16 skinny 16x28672x8192 NN, B stored K x N (HBM bound)"),
    "S16_f32_kn": Workload("S16_f32_kn", F32, 16, 28672, 8192, 0, 0, 1.0, 0.0, "normal", 0.02, 16,
                           "fp32 skinny 16x28672x8192 NN, B stored K x N (HBM bound)"),
    # fp32 with four 16-row blocks: bound by the fp32 MFMA rate, not by HBM
    "S64_f32": Workload("S64_f32", F32, 64, 16384, 8192, 0, 1, 1.0, 0.0, "normal", 0.02, 20,
                        "fp32 skinny 64x16384x8192 NT (fp32 MFMA bound)"),
    # ... and with the small operand stored K x M (the streaming kernels read a copy written out along K)
    "S32_f16_tn": Workload("S32_f16_tn", F16, 32, 28672, 8192, 1, 0, 1.0, 0.0, "normal", 0.02, 18,
                           "f16 skinny 32x28672x8192 TN, A stored K x M, B stored K x N (HBM bound)"),
    "S16_bf16_tt": Workload("S16_bf16_tt", BF16, 16, 16384, 16384, 1, 1, 1.0, 0.0, "normal", 0.02, 19,
                            "bf16 skinny 16x16384x16384 TT, A stored K x M (HBM bound)"),
    # one row of 128 x 128 tiles, B streamed from HBM by the tiled kernel (128 k per stage)
    "D128_bf16": Workload("D128_bf16", BF16, 128, 28672, 8192, 0, 1, 1.0, 0.0, "normal", 0.02, 17,
                          "bf16 128x28672x8192 NT (one row of tiles, HBM bound)"),
    # the two layouts with A stored K x M, as context for the [k][m] staging path
    "T4k_bf16_tn": Workload("T4k_bf16_tn", BF16, 4096, 4096, 4096, 1, 0, 1.0, 0.0, "normal", 1.0 / math.sqrt(4096.0), 9,
                            "bf16 4096^3 TN (A stored K x M, B stored K x N)"),
    "T4k_bf16_tt": Workload("T4k_bf16_tt", BF16, 4096, 4096, 4096, 1, 1, 1.0, 0.0, "normal", 1.0 / math.sqrt(4096.0), 10,
                            "bf16 4096^3 TT (A stored K x M, B stored N x K)"),
}


def bias_vector(seed: int, length: int, ints: bool = False, scale: float = 1.0) -> np.ndarray:
    """fp32 bias of the fused output step (stream 3 of the seed): U[-scale, scale),
    or small integers in [-4, 4] when ``ints``."""
    if ints:
        return small_int_matrix(seed, 3, 1, length, -4, 4, F32).reshape(length).copy()
    return logical_matrix(seed, 3, 1, length, "uniform", scale, F32).reshape(length).copy()


def small_int_matrix(seed: int, stream: int, rows: int, cols: int, lo: int, hi: int, dtype: int) -> np.ndarray:
    """Integer-valued logical matrix with entries in [lo, hi] (exact in every dtype
    for |v| <= 256)."""
    x = raw_bits(seed, stream, 0, rows * cols)
    span = np.uint64(hi - lo + 1)
    v = ((x >> np.uint64(33)) % span).astype(np.int64) + lo
    return round_to_dtype(v.astype(np.float32), dtype).reshape(rows, cols)
