"""16-bit operands with C stored as fp32 (PEAK_GEMM_C_F32): the accumulators reach
memory unrounded, so the fp32 tolerance applies; integers must match exactly."""
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


def _operands(seed, dtype, M, N, K, ta, tb, ints, ldc_pad):
    if ints:
        la = pi.small_int_matrix(seed, 0, M, K, -2, 2, dtype)
        lb = pi.small_int_matrix(seed, 1, K, N, -2, 2, dtype)
        lc = pi.small_int_matrix(seed, 2, M, N, -9, 9, pi.F32)
    else:
        la = pi.logical_matrix(seed, 0, M, K, "normal", 1.0 / np.sqrt(K), dtype)
        lb = pi.logical_matrix(seed, 1, K, N, "normal", 1.0, dtype)
        lc = pi.logical_matrix(seed, 2, M, N, "uniform", 1.0, pi.F32)
    return pi.store(la, bool(ta)), pi.store(lb, bool(tb)), pi.store(lc, False, N + ldc_pad)


# (M, N, K, transA, transB, forced split): interior and edge tiles, odd ldc, K split, the streaming kernels
CASES = [(256, 256, 64, 0, 1, None), (300, 520, 64, 0, 0, None), (136, 72, 48, 1, 0, None), (72, 264, 64, 1, 1, None),
         (260, 264, 64, 0, 1, 2), (16, 192, 64, 0, 1, None), (5, 130, 64, 0, 1, 2)]


@pytest.mark.parametrize("dtype", [pi.F16, pi.BF16])
def test_fp32_c_exact_integers(gu, oracle, dtype):
    pg = gu.pg
    for case, (M, N, K, ta, tb, split) in enumerate(CASES):
        A, B, C = _operands(8000 + case, dtype, M, N, K, ta, tb, True, case % 2 * 3)
        for alpha, beta in [(1.0, 0.0), (-1.0, 2.0)]:
            C0 = C if beta != 0 else gu.nan_fill(C.shape[0], C.shape[1], pi.F32)
            ref = oracle.gemm(dtype, ta, tb, M, N, K, alpha, A, B, beta, C if beta != 0 else None, cdtype=pi.F32)
            got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, alpha, beta, A, B, C0,
                                         flags=pg.force_flags(split=split), cdtype=pi.F32)
            assert raw.dtype == np.float32
            assert np.array_equal(got, ref), (info, M, N, K, alpha, beta)
            assert np.array_equal(raw[:, N:].view(np.uint8), C0[:, N:].view(np.uint8))


@pytest.mark.parametrize("dtype", [pi.F16, pi.BF16])
def test_fp32_c_random_keeps_fp32_accuracy(gu, oracle, dtype):
    pg = gu.pg
    for case, (M, N, K, ta, tb) in enumerate([(384, 320, 512, 0, 1), (513, 259, 1000, 0, 0), (13, 1000, 4096, 0, 1)]):
        A, B, C = _operands(8100 + case, dtype, M, N, K, ta, tb, False, 0)
        ref = oracle.gemm(dtype, ta, tb, M, N, K, 0.75, A, B, -0.5, C, cdtype=pi.F32)
        got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, 0.75, -0.5, A, B, C, cdtype=pi.F32)
        err = oracle.rel_frobenius(got, ref)
        assert err <= gu.TOL[pi.F32], (info, M, N, K, err)      # 1e-5: nothing is rounded to 16 bits
        # with a fused step on top
        bias = pi.bias_vector(8200 + case, N, scale=0.5)
        ref2 = oracle.bias_act(ref, M, pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_GELU_TANH)
        got2, _, info = gu.run_gemm(dtype, ta, tb, M, N, K, 0.75, -0.5, A, B, C, cdtype=pi.F32,
                                    fused=(pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_GELU_TANH))
        assert oracle.rel_frobenius(got2, ref2) <= gu.TOL[pi.F32], info


def test_fp32_c_at_full_size_on_sampled_rows(gu, oracle):
    w = pi.WORKLOADS["C3b"]
    A, B, _ = w.make()
    rows = sorted({0, 255, 256, w.M - 1} | {int(x) for x in np.random.default_rng(4).integers(0, w.M, 6)})
    ref = oracle.gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, 0.0, None, rows=rows)
    got, raw, info = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, 0.0, A, B,
                                 gu.nan_fill(w.M, w.N, pi.F32), cdtype=pi.F32)
    err = oracle.rel_frobenius(got[rows], ref)
    print(info, "fp32-C rel Frobenius error on %d rows: %.3e" % (len(rows), err))
    assert np.isfinite(got).all()
    assert err <= gu.TOL[pi.F32], (info, err)


def test_fp32_c_without_a_product_and_misaligned(gu):
    import torch
    pg = gu.pg
    M, N = 24, 40
    C = pi.logical_matrix(8300, 2, M, N, "uniform", 1.0, pi.F32)
    dC = gu.to_dev(C)
    with pg.Plan(M, N, 0, pi.BF16, 0, 1, flags=pg.PEAK_GEMM_C_F32) as plan:
        plan.run(1.0, 0, 0, -2.0, dC.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy(), np.float32(-2.0) * C)
        st = pg.peak_gemm_run(plan.handle, 1.0, 0, 0, -2.0, dC.data_ptr() + 2, 0, 0, 0)     # C must be 4-byte aligned
        assert st == pg.PEAK_ERR_INVALID_ARG
