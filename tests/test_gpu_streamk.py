"""Hybrid stream-K (the Split-K step applied to the last, partial round of tiles):
the tiles of that round are cut into K slices whose fp32 partial tiles a second
kernel sums in slice order.  Checked against the oracle with exact integers
(bitwise) and random data (per-element bound), in all four layouts, with K
ending inside a K tile, beta != 0, the fused output step and fp32 C."""
import re

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


def _flags(pg, dtype, ta, tb, streamk):
    """The 16x16x32 kernel of the layout, by name (the selector may prefer smaller tiles for these sizes)."""
    names = [pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())]
    name = "%s_m256x256w4a3_%s%s" % ("bf16" if dtype == pi.BF16 else "f16", "t" if ta else "n", "t" if tb else "n")
    return pg.force_flags(variant=names.index(name), streamk=streamk)


def _rows_in_every_tile_row(M, bm, per, seed):
    rng = np.random.default_rng(seed)
    rows = {0, M - 1}
    for r0 in range(0, M, bm):
        rows |= {r0 + int(x) for x in rng.integers(0, min(bm, M - r0), size=per)}
    return sorted(rows)


def _operands(seed, dtype, M, N, K, ta, tb, ints):
    if ints:
        la = pi.small_int_matrix(seed, 0, M, K, -1, 1, dtype)
        lb = pi.small_int_matrix(seed, 1, K, N, -1, 1, dtype)
        lc = pi.small_int_matrix(seed, 2, M, N, -3, 3, dtype)
    else:
        la = pi.logical_matrix(seed, 0, M, K, "normal", 1.0 / np.sqrt(K), dtype)
        lb = pi.logical_matrix(seed, 1, K, N, "normal", 1.0, dtype)
        lc = pi.logical_matrix(seed, 2, M, N, "uniform", 1.0, dtype)
    return pi.store(la, bool(ta)), pi.store(lb, bool(tb)), lc


# 17 x 16 tiles of 256 x 256 (the last row and column of tiles ragged): one full round of 256 and 16 tiles over
M, N = 17 * 256 - 104, 16 * 256 - 8


@pytest.mark.parametrize("dtype", [pi.BF16, pi.F16])
@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_stream_k_exact_integers(gu, oracle, dtype, ta, tb):
    import torch
    pg = gu.pg
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("shape chosen for 256 compute units")
    K = 1032                                          # 17 K tiles, the last one 8 deep
    A, B, C = _operands(9500 + 2 * ta + tb, dtype, M, N, K, ta, tb, True)
    rows = _rows_in_every_tile_row(M, 256, 3, 5)
    ref = oracle.gemm(dtype, ta, tb, M, N, K, 1.0, A, B, 1.0, C, rows=rows)
    assert np.abs(ref).max() <= 256
    got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 1.0, A, B, C, flags=_flags(pg, dtype, ta, tb, True))
    assert "streamk=16" in info and re.search(r"_m256x256w4a3_", info), info
    assert np.array_equal(got[rows], ref), (info, int((got[rows] != ref).sum()))
    # the uncut plan gives the same integers everywhere, and the cut one the same bits twice
    plain, _, info0 = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 1.0, A, B, C, flags=_flags(pg, dtype, ta, tb, False))
    assert "streamk=0" in info0
    assert np.array_equal(got, plain)
    again, raw2, _ = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 1.0, A, B, C, flags=_flags(pg, dtype, ta, tb, True))
    assert np.array_equal(raw.view(np.uint8), raw2.view(np.uint8))
    # fp32 C takes the other store path of the reduction
    C32 = pi.to_f64(C, dtype).astype(np.float32)
    got32, _, info32 = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 1.0, A, B, C32, flags=_flags(pg, dtype, ta, tb, True), cdtype=pi.F32)
    assert "streamk=16" in info32
    assert np.array_equal(got32[rows], ref)


@pytest.mark.parametrize("dtype", [pi.BF16, pi.F16])
def test_stream_k_random_data_and_fused_step(gu, oracle, dtype):
    import torch
    pg = gu.pg
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("shape chosen for 256 compute units")
    K = 2048
    for ta, tb in [(0, 1), (0, 0)]:
        A, B, C = _operands(9600 + tb, dtype, M, N, K, ta, tb, False)
        rows = _rows_in_every_tile_row(M, 256, 2, 6)
        got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, 0.75, -0.5, A, B, C, flags=_flags(pg, dtype, ta, tb, True))
        assert "streamk=16" in info and "split=8 " in info, info
        gu.check_against_oracle(oracle, got, dtype, ta, tb, M, N, K, 0.75, A, B, -0.5, C, rows=rows, what=info)
        # fused bias per column + ReLU: applied by the reduction on the cut tiles, by the GEMM kernel elsewhere
        bias = pi.bias_vector(9600, N, scale=0.5)
        plain, bound = gu.elementwise_bound(oracle, dtype, ta, tb, M, N, K, 1.0, A, B, 0.0, None, rows=rows)
        ref = oracle.bias_act(plain, M, oracle.BIAS_PER_COLUMN, bias, oracle.ACT_RELU, rows=rows)
        got, raw, info = gu.run_gemm(dtype, ta, tb, M, N, K, 1.0, 0.0, A, B, gu.nan_fill(M, N, dtype),
                                     flags=_flags(pg, dtype, ta, tb, True), fused=(pg.PEAK_BIAS_PER_COLUMN, bias, pg.PEAK_ACT_RELU))
        assert "streamk=16" in info, info
        assert oracle.rel_frobenius(got[rows], ref) <= gu.TOL[dtype], info
        # ReLU does not stretch distances and |x + b| <= |x| + |b|: the plain product's bound plus the rounding of the bias' share
        gu.assert_elementwise(got[rows], ref, bound + gu.U_OUT[dtype] * np.abs(bias)[None, :].astype(np.float64) + 2.0 ** -23 * np.abs(bias)[None, :], info)
