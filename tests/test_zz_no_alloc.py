"""peak_gemm_run_static: the entry point for callers that cannot allocate or pass
a workspace (the K-split partials, and the copy of an A stored K x M that a
streaming plan makes, go to an array inside the library's device code).  Its output must equal peak_gemm_run's bit for bit (same plan, same
kernels), on two calls in a row, the second on a smaller problem, so that what
the first call left in the shared array is still there when the second runs."""
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


def _case(gu, oracle, dtype, M, N, K, split, seed, transA=0):
    import torch
    pg = gu.pg
    la = pi.logical_matrix(seed, 0, M, K, "normal", 1.0 / np.sqrt(K), dtype)
    lb = pi.logical_matrix(seed, 1, K, N, "normal", 1.0, dtype)
    lc = pi.logical_matrix(seed, 2, M, N, "uniform", 1.0, dtype)
    A, B = pi.store(la, bool(transA)), pi.store(lb, True)
    stream = torch.cuda.current_stream().cuda_stream
    dA, dB = gu.to_dev(A), gu.to_dev(B)
    with pg.Plan(M, N, K, dtype, transA, 1, flags=pg.force_flags(split=split)) as plan:
        info = plan.info()
        assert "split=%d " % split in info, info
        assert info.endswith("acopy=%d" % transA), info
        assert 0 < plan.workspace_bytes <= pg.PEAK_GEMM_STATIC_WORKSPACE_BYTES
        # the existing entry point, workspace from the caller
        dC1 = gu.to_dev(lc)
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
        plan.run(0.75, dA.data_ptr(), dB.data_ptr(), -0.5, dC1.data_ptr(), ws.data_ptr(), plan.workspace_bytes, stream)
        # the new one: no workspace, no allocation
        dC2 = gu.to_dev(lc)
        torch.cuda.synchronize()
        st = pg.peak_gemm_run_static(plan.handle, 0.75, dA.data_ptr(), dB.data_ptr(), -0.5, dC2.data_ptr(), stream)
        assert st == pg.PEAK_OK, pg.peak_status_string(st)
        torch.cuda.synchronize()
    r1, r2 = gu.from_dev(dC1, dtype), gu.from_dev(dC2, dtype)
    assert np.array_equal(r1.view(np.uint8), r2.view(np.uint8)), info
    got = pi.to_f64(np.ascontiguousarray(r2[:M, :N]), dtype)
    gu.check_against_oracle(oracle, got, dtype, transA, 1, M, N, K, 0.75, A, B, -0.5, lc, what=info)


def test_static_workspace_entry_point_two_calls_in_a_row(gu, oracle):
    # first a problem that fills a good part of the array, then a smaller one with another split
    _case(gu, oracle, pi.BF16, 520, 1000, 4096, 8, 31)          # 8 x 520 x 1000 x 4 B = 16.6 MB of partials
    _case(gu, oracle, pi.BF16, 200, 136, 2048, 3, 32)
    _case(gu, oracle, pi.F32, 130, 264, 1024, 4, 33)
    _case(gu, oracle, pi.BF16, 16, 520, 4096, 2, 34)            # streaming kernel with a K split
    _case(gu, oracle, pi.F16, 24, 4104, 2048, 2, 35, transA=1)  # ... on an A stored K x M: partials and the copy of A


def test_static_workspace_entry_point_limits(gu):
    import torch
    pg = gu.pg
    stream = torch.cuda.current_stream().cuda_stream
    # more partials than the array holds: refused, nothing launched, C untouched
    M, N, K = 2048, 2048, 4096
    with pg.Plan(M, N, K, pi.BF16, 0, 1, flags=pg.force_flags(split=4)) as plan:
        assert plan.workspace_bytes > pg.PEAK_GEMM_STATIC_WORKSPACE_BYTES
        a = torch.zeros(M * K, dtype=torch.int16, device="cuda")
        c = torch.full((M * N,), 0x7FC1, dtype=torch.int16, device="cuda")
        st = pg.peak_gemm_run_static(plan.handle, 1.0, a.data_ptr(), a.data_ptr(), 0.0, c.data_ptr(), stream)
        assert st == pg.PEAK_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert bool((c == 0x7FC1).all())
    # a plan without a K split needs no workspace and runs as peak_gemm_run does
    with pg.Plan(256, 256, 512, pi.BF16, 0, 1, flags=pg.force_flags(split=1)) as plan:
        assert plan.workspace_bytes == 0
        a = torch.zeros(256 * 512, dtype=torch.int16, device="cuda")
        c = torch.full((256 * 256,), 0x7FC1, dtype=torch.int16, device="cuda")
        assert pg.peak_gemm_run_static(plan.handle, 1.0, a.data_ptr(), a.data_ptr(), 0.0, c.data_ptr(), stream) == pg.PEAK_OK
        torch.cuda.synchronize()
        assert bool((c == 0).all())
    assert pg.peak_gemm_run_static(None, 1.0, 0, 0, 0.0, 0, 0) == pg.PEAK_ERR_INVALID_ARG
