"""GPU parity of the fused output step, C = act(alpha*op(A)*op(B) + beta*C + bias),
through peak_gemm_run_fused, against the oracle's gemm followed by its bias_act.
Integer cases must match exactly; the rest within the GEMM tolerances."""
import numpy as np
import pytest

import peak_inputs as pi

pytestmark = pytest.mark.gpu

DTYPES = [pi.F32, pi.F16, pi.BF16]


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from tests import gpu_util
    return gpu_util


def _operands(seed, dtype, M, N, K, transA, transB, ints, ldc_pad=0):
    if ints:
        la = pi.small_int_matrix(seed, 0, M, K, -2, 2, dtype)
        lb = pi.small_int_matrix(seed, 1, K, N, -2, 2, dtype)
        lc = pi.small_int_matrix(seed, 2, M, N, -3, 3, dtype)
    else:
        la = pi.logical_matrix(seed, 0, M, K, "normal", 1.0 / np.sqrt(K), dtype)
        lb = pi.logical_matrix(seed, 1, K, N, "normal", 1.0, dtype)
        lc = pi.logical_matrix(seed, 2, M, N, "uniform", 1.0, dtype)
    return pi.store(la, bool(transA)), pi.store(lb, bool(transB)), pi.store(lc, False, N + ldc_pad)


def _named(gu, name):
    for i in range(gu.pg.peak_gemm_variant_count()):
        if gu.pg.peak_gemm_variant_name(i) == name:
            return i
    raise KeyError(name)


# (M, N, K, transA, transB, forced variant by dtype or None, forced split or None)
# the selector's tiled kernel on interior and edge tiles; K split (the reduction kernel
# applies the step); the smallest tile, forced; the streaming kernels for M <= 16
CASES = [
    (256, 256, 64, 0, 1, None, None),
    (300, 520, 64, 0, 0, None, None),
    (130, 72, 48, 1, 0, None, None),
    (260, 264, 64, 0, 1, None, 2),
    (100, 90, 40, 0, 0, {pi.F32: "f32_r64x64_nn", pi.F16: "f16_r64x64_nn", pi.BF16: "bf16_r64x64_nn"}, None),
    (16, 192, 64, 0, 1, None, None),
    (5, 130, 64, 0, 1, None, 2),
]


@pytest.mark.parametrize("dtype", DTYPES)
def test_fused_exact_integers(gu, oracle, dtype):
    """Small integers, integer bias, ReLU: every value is exact in every storage type."""
    pg = gu.pg
    names = {pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())}
    for case, (M, N, K, ta, tb, forced, split) in enumerate(CASES):
        vid = None
        if forced is not None:
            if forced[dtype] not in names:
                continue
            vid = _named(gu, forced[dtype])
        A, B, C = _operands(7000 + case, dtype, M, N, K, ta, tb, ints=True, ldc_pad=case % 2 * 8)
        for kind, act, alpha, beta in [(pg.PEAK_BIAS_PER_COLUMN, pg.PEAK_ACT_RELU, 1.0, 0.0),
                                       (pg.PEAK_BIAS_PER_ROW, pg.PEAK_ACT_NONE, -1.0, 2.0),
                                       (pg.PEAK_BIAS_NONE, pg.PEAK_ACT_RELU, 1.0, -1.0),
                                       (pg.PEAK_BIAS_PER_ROW, pg.PEAK_ACT_RELU, 1.0, 0.0)]:
            bias = None if kind == pg.PEAK_BIAS_NONE else pi.bias_vector(7100 + case, N if kind == pg.PEAK_BIAS_PER_COLUMN else M, ints=True)
            C0 = C if beta != 0 else gu.nan_fill(C.shape[0], C.shape[1], dtype)
            ref = oracle.gemm(dtype, ta, tb, M, N, K, alpha, A, B, beta, C if beta != 0 else None)
            ref = oracle.bias_act(ref, M, kind, bias, act)
            got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, alpha, beta, A, B, C0,
                                         flags=pg.force_flags(variant=vid, split=split), fused=(kind, bias, act))
            assert np.array_equal(got, ref), (info, M, N, K, kind, act, alpha, beta)
            assert np.array_equal(raw[:, N:].view(np.uint8), C0[:, N:].view(np.uint8))


@pytest.mark.parametrize("dtype", DTYPES)
def test_fused_gelu_and_bias_random(gu, oracle, dtype):
    pg = gu.pg
    for case, (M, N, K, ta, tb) in enumerate([(384, 320, 512, 0, 1), (513, 259, 1000, 0, 0), (700, 70, 2048, 1, 1),
                                              (13, 1000, 4096, 0, 1)]):
        A, B, C = _operands(7200 + case, dtype, M, N, K, ta, tb, ints=False)
        for kind in (pg.PEAK_BIAS_PER_COLUMN, pg.PEAK_BIAS_PER_ROW):
            bias = pi.bias_vector(7300 + case, N if kind == pg.PEAK_BIAS_PER_COLUMN else M, scale=0.5)
            ref = oracle.gemm(dtype, ta, tb, M, N, K, 1.0, A, B, 0.5, C)
            ref = oracle.bias_act(ref, M, kind, bias, pg.PEAK_ACT_GELU_TANH)
            got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 0.5, A, B, C,
                                         fused=(kind, bias, pg.PEAK_ACT_GELU_TANH))
            err = oracle.rel_frobenius(got, ref)
            assert err <= gu.TOL[dtype], (info, M, N, K, kind, err)
            if dtype == pi.F32:
                # element by element as well: the hardware exponential must not show
                assert np.max(np.abs(got - ref)) <= 2e-5 * max(1.0, float(np.max(np.abs(ref)))), info


@pytest.mark.parametrize("dtype", DTYPES)
def test_fused_without_a_product(gu, oracle, dtype):
    """alpha == 0 or K == 0: C = act(beta*C + bias); beta == 1 is not a no-op here."""
    import torch
    pg = gu.pg
    M, N, K = 40, 24, 16
    _, _, C = _operands(7400, dtype, M, N, K, 0, 0, ints=True, ldc_pad=4)
    bias = pi.bias_vector(7401, N, ints=True)
    dbias = gu.to_dev(bias)
    stream = torch.cuda.current_stream().cuda_stream
    cin = pi.to_f64(np.ascontiguousarray(C[:, :N]), dtype)
    for Kp, alpha, beta in [(K, 0.0, 1.0), (0, 1.0, -2.0), (K, 0.0, 0.0)]:
        with pg.Plan(M, N, Kp, dtype, 0, 0, max(Kp, 1), N, N + 4) as plan:
            dC = gu.to_dev(C if beta != 0 else gu.nan_fill(M, N + 4, dtype))
            plan.run_fused(alpha, 0, 0, beta, dC.data_ptr(), pg.PEAK_BIAS_PER_COLUMN, dbias.data_ptr(), pg.PEAK_ACT_RELU,
                           0, 0, stream)
            torch.cuda.synchronize()
            raw = gu.from_dev(dC, dtype)
        want = oracle.bias_act(beta * cin if beta != 0 else np.zeros((M, N)), M, pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_RELU)
        assert np.array_equal(pi.to_f64(np.ascontiguousarray(raw[:, :N]), dtype), want), (Kp, alpha, beta)


def test_null_epilogue_is_the_plain_run_and_bad_ones_are_rejected(gu, oracle):
    import torch
    pg = gu.pg
    M, N, K = 200, 136, 256
    A, B, C = _operands(7500, pi.BF16, M, N, K, 0, 1, ints=False)
    plain, raw0, _ = gu.run_gemm(pi.BF16, 0, 1, M, N, K, 1.0, 0.5, A, B, C)
    same, raw1, _ = gu.run_gemm(pi.BF16, 0, 1, M, N, K, 1.0, 0.5, A, B, C, fused=(pg.PEAK_BIAS_NONE, None, pg.PEAK_ACT_NONE))
    assert np.array_equal(raw0.view(np.uint8), raw1.view(np.uint8))
    dA, dB, dC = gu.to_dev(A), gu.to_dev(B), gu.to_dev(C)
    with pg.Plan(M, N, K, pi.BF16, 0, 1) as plan:
        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
        st = pg.peak_gemm_run_fused(plan.handle, 1.0, dA.data_ptr(), dB.data_ptr(), 0.5, dC.data_ptr(), None,
                                    ws.data_ptr(), plan.workspace_bytes, 0)
        assert st == pg.PEAK_OK
        torch.cuda.synchronize()
        assert np.array_equal(gu.from_dev(dC, pi.BF16).view(np.uint8), raw0.view(np.uint8))
        for ep in (pg.PeakGemmEpilogue(None, pg.PEAK_BIAS_PER_ROW, 0), pg.PeakGemmEpilogue(None, 3, 0),
                   pg.PeakGemmEpilogue(None, 0, 7), pg.PeakGemmEpilogue(dA.data_ptr() + 2, pg.PEAK_BIAS_PER_COLUMN, 0)):
            st = pg.peak_gemm_run_fused(plan.handle, 1.0, dA.data_ptr(), dB.data_ptr(), 0.0, dC.data_ptr(), ep,
                                        ws.data_ptr(), plan.workspace_bytes, 0)
            assert st == pg.PEAK_ERR_INVALID_ARG


def test_fused_at_full_size_on_sampled_rows(gu, oracle):
    """bf16 4096^3 in the launch configuration the bench times, bias per column and GELU."""
    pg = gu.pg
    w = pi.WORKLOADS["C3b"]
    A, B, _ = w.make()
    bias = pi.bias_vector(7600, w.N, scale=0.5)
    rows = sorted({0, 255, 256, 2047, w.M - 1} | {int(x) for x in np.random.default_rng(3).integers(0, w.M, 8)})
    ref = oracle.gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, 0.0, None, rows=rows)
    ref = oracle.bias_act(ref, w.M, pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_GELU_TANH, rows=rows)
    got, raw, info = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, 0.0, A, B,
                                 gu.nan_fill(w.M, w.N, w.dtype), fused=(pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_GELU_TANH))
    err = oracle.rel_frobenius(got[rows], ref)
    print(info, "fused rel Frobenius error on %d rows: %.3e" % (len(rows), err))
    assert np.isfinite(got).all()
    assert err <= gu.TOL[w.dtype], (info, err)
