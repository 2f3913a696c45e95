"""Helpers for the GPU parity tests: move seeded host arrays to the device, run
the C-ABI entry points, bring the result back as fp64 values."""
from __future__ import annotations

import numpy as np
import torch

import peak_inputs as pi
import paper_2512_19018_amd as pg

TOL = {pi.F32: 1e-5, pi.F16: 2e-2, pi.BF16: 2e-2}     # relative Frobenius, as stated for the workloads


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
