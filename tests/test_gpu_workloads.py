"""The graded workloads at full size, in the launch configuration the bench
times (the selector's own choice), checked on sampled rows of C that the oracle
computes one by one."""
import numpy as np
import pytest

import peak_inputs as pi

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from tests import gpu_util
    return gpu_util


def _sample_rows(M, count, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, M - 1, M // 2, min(255, M - 1), min(256, M - 1)]
    rows = sorted(set(fixed) | set(int(x) for x in rng.integers(0, M, size=max(0, count - len(fixed)))))
    return rows


@pytest.mark.parametrize("name,nrows", [("C1", 256), ("C2", 12), ("C3", 10), ("C3b", 16), ("C4", 12), ("C5", 16),
                                        ("P2k_f32", 16), ("P2k_f16", 16), ("P4k_f16", 12),
                                        ("T4k_bf16_tn", 12), ("T4k_bf16_tt", 12)])
def test_workload_against_oracle(gu, oracle, name, nrows):
    w = pi.WORKLOADS[name]
    A, B, C = w.make()
    rows = list(range(w.M)) if nrows >= w.M else _sample_rows(w.M, nrows, 7)
    ref = oracle.gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, w.beta, C, rows=rows)
    C0 = C if w.beta != 0 else gu.nan_fill(w.M, w.N, w.dtype)
    got, raw, info = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, w.beta, A, B, C0)
    print(name, info)
    err = oracle.rel_frobenius(got[rows], ref)
    print(name, "rel Frobenius error on %d rows: %.3e" % (len(rows), err))
    assert np.isfinite(got).all()
    assert err <= gu.TOL[w.dtype], (name, info, err)
    # properties that hold at any size: run-to-run bits, and linearity in alpha
    # against a second run with alpha doubled (exact: scaling by 2 commutes with
    # rounding, except where the result is subnormal in the storage type)
    got2, raw2, _ = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, w.beta, A, B, C0)
    assert np.array_equal(raw.view(np.uint8), raw2.view(np.uint8))
    if w.beta == 0:
        got3, _, _ = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, 2.0 * w.alpha, 0.0, A, B, C0)
        normal = np.abs(got) > 1e-3
        assert np.array_equal(got3[normal], 2.0 * got[normal])
