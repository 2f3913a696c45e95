"""The graded workloads at full size, in the launch configuration the bench
times (the selector's own choice), checked on rows of C that the oracle computes
one by one: several rows in every row of tiles of the plan, all columns, each
element against its own bound as well as through the norm."""
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


def _sample_rows(M, info, per_tile_row, seed):
    """Rows of C to check: `per_tile_row` in EVERY row of tiles of the plan (its tile
    height is read from the plan's description), at seeded random heights within the
    tile, plus the first and last row of the matrix and of the first tile.  Every row
    is checked over all N columns, so every output tile of the launch is covered."""
    bm = int(re.search(r"tile=(\d+)x", info).group(1))
    rng = np.random.default_rng(seed)
    rows = {0, M - 1, min(bm - 1, M - 1), min(bm, M - 1)}
    for r0 in range(0, M, bm):
        h = min(bm, M - r0)
        rows |= {r0 + int(x) for x in rng.integers(0, h, size=per_tile_row)}
    return sorted(rows)


# (workload, rows per tile row, forced K split or None for the selector's own plan, which the bench times)
CASES = [("C1", 256, None), ("C2", 2, None), ("C3", 3, None), ("C3b", 3, None), ("C4", 3, None), ("C5", 16, None),
         ("C4", 2, 2), ("C4", 2, 3),
         ("P2k_f32", 2, None), ("P4k_f32", 2, None), ("P2k_f16", 3, None), ("P4k_f16", 3, None),
         ("T4k_bf16_tn", 3, None), ("T4k_bf16_tt", 3, None), ("SK_bf16", 2, None),
         # the streaming path beyond M <= 16 / 16 bits / B along K: every row
         ("S32_bf16", 32, None), ("S64_f16", 64, None), ("S16_f32", 16, None), ("S16_bf16_kn", 16, None),
         ("S16_f32_kn", 16, None), ("S64_f32", 64, None),
         # ... and with A stored K x M: the run writes A out along K first
         ("S32_f16_tn", 32, None), ("S16_bf16_tt", 16, None),
         # one row of tiles of the 16x16x32 kernels: workgroups start at different K tiles
         ("D128_bf16", 24, None)]


@pytest.mark.parametrize("name,per_tile_row,split", CASES)
def test_workload_against_oracle(gu, oracle, name, per_tile_row, split):
    w = pi.WORKLOADS[name]
    A, B, C = w.make()
    flags = gu.pg.force_flags(split=split)
    C0 = C if w.beta != 0 else gu.nan_fill(w.M, w.N, w.dtype)
    got, raw, info = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, w.beta, A, B, C0, flags=flags)
    print(name, info)
    if name.startswith("S") and name != "SK_bf16":
        assert "skinny" in info, info
    if name in ("S32_f16_tn", "S16_bf16_tt"):
        assert info.endswith("acopy=1"), info
    if name == "D128_bf16":
        assert "_m128x128" in info and " rot=0,1 " in info, info
    if split is not None:
        assert "split=%d" % split in info, info
    rows = _sample_rows(w.M, info, per_tile_row, 7)
    err = gu.check_against_oracle(oracle, got, w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, w.beta, C,
                                  rows=rows, what=(name, info))
    print(name, "rel Frobenius error on %d rows (every tile row of the plan): %.3e" % (len(rows), err))
    assert np.isfinite(got).all()
    # properties that hold at any size: run-to-run bits, and linearity in alpha
    # against a second run with alpha doubled (exact: scaling by 2 commutes with
    # rounding, except where the result is subnormal in the storage type)
    got2, raw2, _ = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, w.beta, A, B, C0, flags=flags)
    assert np.array_equal(raw.view(np.uint8), raw2.view(np.uint8))
    if w.beta == 0:
        got3, _, _ = gu.run_gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, 2.0 * w.alpha, 0.0, A, B, C0, flags=flags)
        normal = np.abs(got) > 1e-3
        assert np.array_equal(got3[normal], 2.0 * got[normal])
