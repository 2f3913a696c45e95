"""Helpers for the GPU parity tests: move seeded host arrays to the device, run
the C-ABI entry points, bring the result back as fp64 values."""
from __future__ import annotations

import numpy as np
import torch

import peak_inputs as pi
import paper_2512_19018_amd as pg

TOL = {pi.F32: 1e-5, pi.F16: 2e-2, pi.BF16: 2e-2}     # relative Frobenius, as stated for the workloads

# Unit roundoff of the one rounding to the storage type of C (round to nearest even).
U_OUT = {pi.F32: 2.0 ** -24, pi.F16: 2.0 ** -11, pi.BF16: 2.0 ** -8}


def abs_stored(arr: np.ndarray) -> np.ndarray:
    """|x| of a stored array (16-bit types are bit patterns: clear the sign)."""
    if arr.dtype == np.uint16:
        return arr & np.uint16(0x7FFF)
    return np.abs(arr)


def elementwise_bound(oracle, dtype, transA, transB, M, N, K, alpha, A, B, beta, C, rows=None, cdtype=None):
    """Per-element error bound of an fp32-accumulating GEMM against the exact result.

    With S = |alpha| * sum_k |a_ik||b_kj| + |beta||c_ij| (computed by the oracle on the
    absolute values), any order of fp32 additions of the K products, each addition and
    each product rounded with relative error <= 2^-23 (the matrix cores may truncate
    where IEEE would round to nearest, hence not 2^-24), plus the scalings by alpha and
    beta, gives |acc - exact| <= (K + 8) * 2^-23 * S to first order.  The one rounding to
    the storage type of C adds u_out * |value|.  Returns the array of bounds
        u_out * |ref| + (1 + u_out) * (K + 8) * 2^-23 * S
    (shape of the oracle's result for `rows`); `ref` itself is returned alongside."""
    ref = oracle.gemm(dtype, transA, transB, M, N, K, alpha, A, B, beta, C if beta != 0 else None, rows=rows,
                      **({"cdtype": cdtype} if cdtype is not None else {}))
    Cabs = abs_stored(C) if (beta != 0 and C is not None) else None
    S = oracle.gemm(dtype, transA, transB, M, N, K, abs(alpha), abs_stored(A), abs_stored(B), abs(beta), Cabs,
                    rows=rows, **({"cdtype": cdtype} if cdtype is not None else {}))
    out_dt = cdtype if cdtype is not None else dtype
    u = U_OUT[out_dt]
    floor = 2.0 ** -25 if out_dt == pi.F16 else 0.0          # half the smallest f16 subnormal
    return ref, u * np.abs(ref) + (1.0 + u) * (K + 8) * 2.0 ** -23 * S + floor


def assert_elementwise(got, ref, bound, what):
    """Every element within its own bound; reports the worst offender."""
    assert np.isfinite(got).all(), ("non-finite output", what)
    excess = np.abs(got - ref) - bound
    if (excess > 0).any():
        i = np.unravel_index(np.argmax(excess), excess.shape)
        raise AssertionError("%s: element %s got %r ref %r bound %.3e (%d of %d elements out of bound)"
                             % (what, i, got[i], ref[i], bound[i], int((excess > 0).sum()), excess.size))


def to_dev(arr: np.ndarray) -> torch.Tensor:
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def from_dev(t: torch.Tensor, dtype: int) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint16) if dtype != pi.F32 else a


def nan_fill(rows: int, cols: int, dtype: int) -> np.ndarray:
    if dtype == pi.F32:
        return np.full((rows, cols), np.nan, dtype=np.float32)
    return np.full((rows, cols), 0x7FC1 if dtype == pi.BF16 else 0x7E01, dtype=np.uint16)


def check_against_oracle(oracle, got, dtype, transA, transB, M, N, K, alpha, A, B, beta, C, rows=None, cdtype=None,
                         what=""):
    """got: the GPU's values as fp64, [M, N] (all rows; `rows` selects those the oracle
    computes).  Asserts the stated relative Frobenius tolerance AND the per-element
    bound; returns the Frobenius error."""
    from oracle import gemm_oracle
    ref, bound = elementwise_bound(oracle, dtype, transA, transB, M, N, K, alpha, A, B, beta, C, rows, cdtype)
    g = got if rows is None else got[np.asarray(rows, dtype=np.int64)]
    err = gemm_oracle.rel_frobenius(g, ref)
    assert err <= TOL[cdtype if cdtype is not None else dtype], (what, err)
    assert_elementwise(g, ref, bound, what)
    return err


def run_gemm(dtype, transA, transB, M, N, K, alpha, beta, A, B, C0, flags=0, repeat=1, a_off=0, b_off=0,
             fused=None, cdtype=None):
    """A, B, C0: stored host arrays (2-D; row length = leading dimension).  C0 is
    the initial content of C (C_in, or a NaN fill when beta == 0).  ``fused``:
    None for peak_gemm_run, or (bias_kind, fp32 bias array or None, act) for
    peak_gemm_run_fused.  ``cdtype``: storage type of C0 when it is not that of
    A and B (sets PEAK_GEMM_C_F32).  Returns (C values as fp64 [M, N], raw stored C after
    the run, plan info)."""
    lda, ldb, ldc = A.shape[1], B.shape[1], C0.shape[1]
    dA, dB, dC = to_dev(A), to_dev(B), to_dev(C0)
    stream = torch.cuda.current_stream().cuda_stream
    if cdtype is not None and cdtype != dtype:
        assert cdtype == pi.F32
        flags |= pg.PEAK_GEMM_C_F32
    else:
        cdtype = dtype
    with pg.Plan(M, N, K, dtype, transA, transB, lda, ldb, ldc, flags) as plan:
        info = plan.info()
        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
        dbias = to_dev(fused[1]) if fused is not None and fused[1] is not None else None
        for _ in range(repeat):
            if fused is None:
                plan.run(alpha, dA.data_ptr() + a_off, dB.data_ptr() + b_off, beta, dC.data_ptr(),
                         ws.data_ptr(), plan.workspace_bytes, stream)
            else:
                plan.run_fused(alpha, dA.data_ptr() + a_off, dB.data_ptr() + b_off, beta, dC.data_ptr(),
                               fused[0], dbias.data_ptr() if dbias is not None else 0, fused[2],
                               ws.data_ptr(), plan.workspace_bytes, stream)
        torch.cuda.synchronize()
    raw = from_dev(dC, cdtype)
    vals = pi.to_f64(np.ascontiguousarray(raw[:M, :N]), cdtype) if M and N else np.zeros((M, N))
    return vals, raw, info


def variants_for(dtype, transA, transB):
    """ids of all variants built for this dtype and layout."""
    pre = {pi.F32: "f32_", pi.F16: "f16_", pi.BF16: "bf16_"}[dtype]
    suf = "_" + ("t" if transA else "n") + ("t" if transB else "n")
    out = []
    for i in range(pg.peak_gemm_variant_count()):
        n = pg.peak_gemm_variant_name(i)
        if n.startswith(pre) and n.endswith(suf):
            out.append((i, n))
    return out
