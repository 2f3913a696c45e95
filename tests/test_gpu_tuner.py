"""The offline sweep and the selector table, end to end on the GPU."""
import pytest

import peak_inputs as pi

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from tests import gpu_util
    return gpu_util


def test_sweep_writes_a_table_the_library_follows(gu, oracle, tmp_path):
    from paper_2512_19018_amd import tune
    pg = gu.pg
    dtype, tA, tB, M, N, K = pi.BF16, 0, 1, 384, 512, 2048
    res = tune.sweep(dtype, tA, tB, M, N, K, reps=5, warmup=2)
    assert len(res) >= 10 and all(us > 0 for us, _, _ in res)
    assert [r[0] for r in res] == sorted(r[0] for r in res)
    us, name, split = res[0]
    table = tmp_path / "table.txt"
    table.write_text(tune.table_line(dtype, tA, tB, M, N, K, name, split, us) + "\n")
    try:
        assert pg.peak_gemm_load_tuning(str(table)) == 1
        with pg.Plan(M, N, K, dtype, tA, tB) as p:
            assert name in p.info() and ("split=%d " % split) in p.info()
        # and the tabled choice computes the right product
        A = pi.store(pi.logical_matrix(31, 0, M, K, "uniform", 1.0, dtype), tA)
        B = pi.store(pi.logical_matrix(31, 1, K, N, "uniform", 1.0, dtype), tB)
        C0 = gu.nan_fill(M, N, dtype)
        ref = oracle.gemm(dtype, tA, tB, M, N, K, 1.0, A, B, 0.0, None)
        got, raw, info = gu.run_gemm(dtype, tA, tB, M, N, K, 1.0, 0.0, A, B, C0)
        assert name in info
        assert oracle.rel_frobenius(got, ref) <= gu.TOL[dtype]
    finally:
        pg.peak_gemm_load_tuning(None)
