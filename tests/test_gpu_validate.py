"""The library's own correctness validator (guard bands, NaN-poisoned C, two runs,
agreement with the plainest variant) must find nothing on the shipped kernels."""
import pytest

import paper_2512_19018_amd as pg
from paper_2512_19018_amd import validate as val

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,ta,tb,M,N,K,beta,samples", [
    (pg.PEAK_DT_BF16, 0, 1, 300, 520, 1000, 0.0, None),       # every accepted variant and split
    (pg.PEAK_DT_F16, 0, 0, 264, 328, 520, 0.5, 24),
    (pg.PEAK_DT_F32, 1, 0, 200, 136, 300, 0.0, 16),
    (pg.PEAK_DT_BF16, 0, 1, 16, 1024, 2048, 0.0, None),       # the streaming kernels
])
def test_validator_is_clean(dtype, ta, tb, M, N, K, beta, samples):
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    lines = []
    failures = val.validate(dtype, ta, tb, M, N, K, 1.0, beta, samples, seed=3, log=lines.append)
    print("\n".join(lines))
    assert len(lines) >= 2
    assert failures == []
