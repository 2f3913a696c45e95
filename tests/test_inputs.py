"""The seeded generator: determinism, independence of chunking, ranges and the
rounding to the storage types."""
import numpy as np
import torch

import peak_inputs as pi


def test_counter_based_and_chunk_independent():
    whole = pi.raw_bits(7, 1, 0, 1000)
    parts = np.concatenate([pi.raw_bits(7, 1, 0, 333), pi.raw_bits(7, 1, 333, 667)])
    assert (whole == parts).all()
    assert (pi.raw_bits(7, 1, 0, 16) != pi.raw_bits(7, 0, 0, 16)).all()
    assert (pi.raw_bits(8, 1, 0, 16) != pi.raw_bits(7, 1, 0, 16)).all()


def test_splitmix_finaliser_scalar_model():
    # the same arithmetic with Python integers
    def mix(z):
        z &= (1 << 64) - 1
        z ^= z >> 30
        z = (z * 0xBF58476D1CE4E5B9) & ((1 << 64) - 1)
        z ^= z >> 27
        z = (z * 0x94D049BB133111EB) & ((1 << 64) - 1)
        z ^= z >> 31
        return z
    seed, stream = 3, 2
    base = mix(seed * 0x9E3779B97F4A7C15 + (stream + 1) * 0xD1B54A32D192ED03)
    want = [mix(base + (e + 1) * 0x9E3779B97F4A7C15) for e in range(5, 9)]
    got = pi.raw_bits(seed, stream, 5, 4)
    assert [int(x) for x in got] == want


def test_uniform_range_and_moments():
    m = pi.logical_matrix(0, 0, 512, 512, "uniform", 1.0, pi.F32)
    assert m.dtype == np.float32 and m.min() >= -1.0 and m.max() < 1.0
    assert abs(float(m.mean())) < 0.01
    assert abs(float(m.var()) - 1.0 / 3.0) < 0.01


def test_normal_moments_and_scale():
    m = pi.logical_matrix(2, 1, 512, 512, "normal", 0.02, pi.F32)
    assert abs(float(m.mean())) < 1e-3
    assert abs(float(m.std()) - 0.02) < 5e-4


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(200000).astype(np.float32) * np.float32(3.0)
    v[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40]
    ours = pi.f32_to_bf16_bits(v)
    theirs = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (ours == theirs).all()
    back = pi.bf16_bits_to_f32(ours)
    assert (back == torch.from_numpy(v).to(torch.bfloat16).float().numpy()).all()


def test_storage_layout_and_padding():
    lg = pi.small_int_matrix(1, 0, 5, 7, -3, 3, pi.BF16)
    st = pi.store(lg, trans=True, ld=9)
    assert st.shape == (7, 9)
    assert (st[:, :5] == lg.T).all()
    assert (st[:, 5:] == 0x7FC1).all()


def test_workload_table_matches_the_configs():
    w = pi.WORKLOADS
    assert (w["C1"].M, w["C1"].N, w["C1"].K, w["C1"].dtype) == (256, 256, 256, pi.F32)
    assert (w["C2"].alpha, w["C2"].beta, w["C2"].seed) == (1.0, 0.5, 1)
    assert (w["C3"].transA, w["C3"].transB, w["C3"].dtype, w["C3"].K) == (0, 1, pi.BF16, 8192)
    assert (w["C4"].M, w["C4"].N, w["C4"].K, w["C4"].dtype) == (5000, 3000, 12288, pi.F16)
    assert (w["C5"].M, w["C5"].N, w["C5"].K, w["C5"].transB) == (16, 16384, 16384, 1)
    assert w["C5"].min_bytes == (16 * 16384 + 16384 * 16384 + 16 * 16384) * 2
