"""Pins for the CPU oracle: things the mathematics fixes, none of which come
from the oracle itself or from the GPU path.

Each pin is aimed at a plausible mistake: a transposed operand, a wrong
leading dimension, a dropped or mis-scaled beta term, alpha applied to the
wrong term, reading C_in when beta == 0, a wrong element decoder, a k loop
that stops short, a row subset that is mis-indexed.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import peak_inputs as pi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DTYPES = [pi.F32, pi.F16, pi.BF16]


def _int_values(stored, dtype):
    return np.rint(pi.to_f64(stored, dtype)).astype(np.int64)


def _brute_int(transA, transB, M, N, K, alpha, a, lda, b, ldb, beta, c, ldc):
    """int64 triple loop straight on the flat stored arrays."""
    out = [[0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                av = a[k * lda + i] if transA else a[i * lda + k]
                bv = b[j * ldb + k] if transB else b[k * ldb + j]
                s += int(av) * int(bv)
            out[i][j] = alpha * s + (beta * int(c[i * ldc + j]) if beta != 0 else 0)
    return np.array(out, dtype=np.int64).reshape(M, N)


SHAPES = [(1, 1, 1), (2, 3, 5), (7, 5, 3), (13, 17, 11), (4, 1, 9), (1, 6, 2), (16, 8, 17), (3, 3, 1)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("transA,transB", list(itertools.product([0, 1], [0, 1])))
def test_exact_integer_brute_force(oracle, dtype, transA, transB):
    case = 0
    for (M, N, K) in SHAPES:
        for alpha, beta in [(1, 0), (-2, 1), (3, -1), (0, 2), (1, 2)]:
            case += 1
            seed = 100 + case
            la = pi.small_int_matrix(seed, 0, M, K, -3, 3, dtype)
            lb = pi.small_int_matrix(seed, 1, K, N, -3, 3, dtype)
            lc = pi.small_int_matrix(seed, 2, M, N, -3, 3, dtype)
            pad = case % 3            # leading dimensions above the minimum
            A = pi.store(la, bool(transA), (M if transA else K) + pad)
            B = pi.store(lb, bool(transB), (K if transB else N) + 2 * pad)
            C = pi.store(lc, False, N + pad)
            # padding carries NaN patterns: reading it would poison the result
            fa = np.nan_to_num(pi.to_f64(A, dtype), nan=99.0).astype(np.int64).ravel()
            fb = np.nan_to_num(pi.to_f64(B, dtype), nan=99.0).astype(np.int64).ravel()
            fc = np.nan_to_num(pi.to_f64(C, dtype), nan=99.0).astype(np.int64).ravel()
            want = _brute_int(transA, transB, M, N, K, alpha, fa, A.shape[1], fb, B.shape[1],
                              beta, fc, C.shape[1])
            for order in (0, 1):
                got = oracle.gemm(dtype, transA, transB, M, N, K, float(alpha), A, B,
                                  float(beta), C, order=order, threads=1 + case % 3)
                assert np.array_equal(got, want.astype(np.float64)), (M, N, K, alpha, beta, order)


def test_hand_worked_example(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "hand_product_3x4x2.txt"))
            if l.strip() and not l.startswith("#")]
    vals = [[float(x) for x in r] for r in rows]
    A = np.array(vals[0:3], dtype=np.float32)
    B = np.array(vals[3:7], dtype=np.float32)
    C = np.array(vals[7:10], dtype=np.float64)
    Cin = np.array(vals[10:13], dtype=np.float32)
    out = np.array(vals[13:16], dtype=np.float64)
    assert np.array_equal(oracle.gemm(pi.F32, 0, 0, 3, 2, 4, 1.0, A, B), C)
    assert np.array_equal(oracle.gemm(pi.F32, 0, 0, 3, 2, 4, 2.0, A, B, -1.0, Cin), out)
    # the same numbers in the 16-bit storages
    for dt in (pi.F16, pi.BF16):
        got = oracle.gemm(dt, 0, 0, 3, 2, 4, 2.0, pi.round_to_dtype(A, dt).reshape(A.shape),
                          pi.round_to_dtype(B, dt).reshape(B.shape), -1.0,
                          pi.round_to_dtype(Cin, dt).reshape(Cin.shape))
        assert np.array_equal(got, out)


@pytest.mark.parametrize("dtype", DTYPES)
def test_identity_and_permutation(oracle, dtype):
    M, K = 37, 29
    la = pi.logical_matrix(11, 0, M, K, "uniform", 1.0, dtype)
    eye = pi.round_to_dtype(np.eye(K, dtype=np.float32), dtype).reshape(K, K)
    got = oracle.gemm(dtype, 0, 0, M, K, K, 1.0, la, eye)
    assert np.array_equal(got, pi.to_f64(la, dtype))                     # A * I = A
    perm = np.random.default_rng(5).permutation(K)
    P = np.zeros((K, K), dtype=np.float32)
    P[perm, np.arange(K)] = 1.0                                          # column j of A*P is column perm[j] of A
    Pst = pi.round_to_dtype(P, dtype).reshape(K, K)
    got = oracle.gemm(dtype, 0, 0, M, K, K, 1.0, la, Pst)
    assert np.array_equal(got, pi.to_f64(la, dtype)[:, perm])
    # the same permutation handed over transposed
    got = oracle.gemm(dtype, 0, 1, M, K, K, 1.0, la, np.ascontiguousarray(Pst.T))
    assert np.array_equal(got, pi.to_f64(la, dtype)[:, perm])
    # row permutation through A
    Q = np.zeros((M, M), dtype=np.float32)
    rperm = np.random.default_rng(6).permutation(M)
    Q[np.arange(M), rperm] = 1.0
    got = oracle.gemm(dtype, 0, 0, M, K, M, 1.0, pi.round_to_dtype(Q, dtype).reshape(M, M), la)
    assert np.array_equal(got, pi.to_f64(la, dtype)[rperm, :])


@pytest.mark.parametrize("dtype", DTYPES)
def test_closed_forms(oracle, dtype):
    # ones * ones = K everywhere
    M, N, K = 9, 14, 200
    one = lambda r, c: pi.round_to_dtype(np.ones((r, c), np.float32), dtype).reshape(r, c)
    assert np.array_equal(oracle.gemm(dtype, 0, 0, M, N, K, 1.0, one(M, K), one(K, N)),
                          np.full((M, N), float(K)))
    # rank one: (u 1^T)(1 v^T) = K u v^T
    u = np.arange(-4, 5, dtype=np.float32)[:M].reshape(M, 1)
    v = np.arange(-6, 8, dtype=np.float32)[:N].reshape(1, N)
    A = pi.round_to_dtype(np.repeat(u, K, axis=1), dtype).reshape(M, K)
    B = pi.round_to_dtype(np.repeat(v, K, axis=0), dtype).reshape(K, N)
    assert np.array_equal(oracle.gemm(dtype, 0, 0, M, N, K, 1.0, A, B),
                          float(K) * (u.astype(np.float64) @ v.astype(np.float64)))
    # A[i][k] = i + k, B[k][j] = k - j:
    #   C[i][j] = sum_k (i+k)(k-j) = S2 + (i-j) S1 - i j K  with S1 = K(K-1)/2, S2 = (K-1)K(2K-1)/6
    M, N, K = 6, 5, 12
    i = np.arange(M).reshape(M, 1)
    j = np.arange(N).reshape(1, N)
    k = np.arange(K)
    A = pi.round_to_dtype((i + k.reshape(1, K)).astype(np.float32), dtype).reshape(M, K)
    B = pi.round_to_dtype((k.reshape(K, 1) - j).astype(np.float32), dtype).reshape(K, N)
    S1, S2 = K * (K - 1) // 2, (K - 1) * K * (2 * K - 1) // 6
    want = (S2 + (i - j) * S1 - i * j * K).astype(np.float64)
    assert np.array_equal(oracle.gemm(dtype, 0, 0, M, N, K, 1.0, A, B), want)
    # geometric rows: A[i][k] = 2^-k, B[k][j] = 2^k  ->  C = K  (all terms exactly 1)
    K = 14
    k = np.arange(K)
    A = pi.round_to_dtype(np.tile((0.5 ** k[:K]).astype(np.float32), (3, 1)), dtype).reshape(3, K)
    B = pi.round_to_dtype(np.tile((2.0 ** k[:K]).astype(np.float32).reshape(K, 1), (1, 4)), dtype).reshape(K, 4)
    assert np.array_equal(oracle.gemm(dtype, 0, 0, 3, 4, K, 1.0, A, B), np.full((3, 4), float(K)))


def test_rotation_product(oracle):
    # R(a) R(b) = R(a + b), to fp32 input rounding
    a, b = 0.3, 1.1
    R = lambda t: np.array([[np.cos(t), -np.sin(t)], [np.sin(t), np.cos(t)]], dtype=np.float32)
    got = oracle.gemm(pi.F32, 0, 0, 2, 2, 2, 1.0, R(a), R(b))
    assert np.allclose(got, R(a + b).astype(np.float64), atol=3e-7)


@pytest.mark.parametrize("dtype", DTYPES)
def test_transpose_identity_and_flag_equivalence(oracle, dtype):
    M, N, K = 23, 31, 45
    la = pi.logical_matrix(21, 0, M, K, "normal", 1.0, dtype)
    lb = pi.logical_matrix(21, 1, K, N, "normal", 1.0, dtype)
    base = oracle.gemm(dtype, 0, 0, M, N, K, 1.0, la, lb)
    # every flag combination on re-laid-out storage gives the same bits
    for tA, tB in itertools.product([0, 1], [0, 1]):
        got = oracle.gemm(dtype, tA, tB, M, N, K, 1.0, pi.store(la, bool(tA), (M if tA else K) + 3),
                          pi.store(lb, bool(tB), (K if tB else N) + 5))
        assert np.array_equal(got, base), (tA, tB)
    # (A B)^T = B^T A^T : swap the roles; stored B read as "A^T" etc.
    gt = oracle.gemm(dtype, 1, 1, N, M, K, 1.0, lb, la)          # op(A') = lb^T (N x K), op(B') = la^T (K x M)
    assert np.array_equal(gt, base.T)


@pytest.mark.parametrize("dtype", DTYPES)
def test_linearity_in_alpha_beta(oracle, dtype):
    M, N, K = 19, 27, 64
    la = pi.logical_matrix(31, 0, M, K, "uniform", 1.0, dtype)
    lb = pi.logical_matrix(31, 1, K, N, "uniform", 1.0, dtype)
    lc = pi.logical_matrix(31, 2, M, N, "uniform", 1.0, dtype)
    prod = oracle.gemm(dtype, 0, 0, M, N, K, 1.0, la, lb)
    for alpha, beta in [(0.75, 0.5), (-1.25, 2.0), (0.0, 1.5), (2.0, 0.0), (0.1, -0.3)]:
        a32, b32 = float(np.float32(alpha)), float(np.float32(beta))
        got = oracle.gemm(dtype, 0, 0, M, N, K, alpha, la, lb, beta, lc)
        want = a32 * prod + b32 * pi.to_f64(lc, dtype)
        assert np.allclose(got, want, rtol=0, atol=4 * np.finfo(np.float64).eps * (np.abs(want).max() + 1))
    # additivity on integer data, exactly
    a1 = pi.small_int_matrix(41, 0, M, K, -3, 3, dtype)
    a2 = pi.small_int_matrix(42, 0, M, K, -3, 3, dtype)
    bb = pi.small_int_matrix(41, 1, K, N, -3, 3, dtype)
    s = pi.round_to_dtype((pi.to_f64(a1, dtype) + pi.to_f64(a2, dtype)).astype(np.float32), dtype).reshape(M, K)
    assert np.array_equal(oracle.gemm(dtype, 0, 0, M, N, K, 1.0, s, bb),
                          oracle.gemm(dtype, 0, 0, M, N, K, 1.0, a1, bb)
                          + oracle.gemm(dtype, 0, 0, M, N, K, 1.0, a2, bb))


def test_beta_zero_ignores_cin_and_alpha_zero_ignores_operands(oracle):
    M, N, K = 5, 6, 7
    la = pi.logical_matrix(51, 0, M, K, "uniform", 1.0, pi.F32)
    lb = pi.logical_matrix(51, 1, K, N, "uniform", 1.0, pi.F32)
    nanc = np.full((M, N), np.nan, dtype=np.float32)
    got = oracle.gemm(pi.F32, 0, 0, M, N, K, 1.0, la, lb, 0.0, nanc)
    assert np.isfinite(got).all()
    nana = np.full((M, K), np.nan, dtype=np.float32)
    lc = pi.logical_matrix(51, 2, M, N, "uniform", 1.0, pi.F32)
    got = oracle.gemm(pi.F32, 0, 0, M, N, K, 0.0, nana, lb, 2.0, lc)
    assert np.array_equal(got, 2.0 * lc.astype(np.float64))
    # K == 0: C = beta * C_in
    got = oracle.gemm(pi.F32, 0, 0, M, N, 0, 1.0, np.zeros((M, 1), np.float32), np.zeros((1, N), np.float32), -1.0, lc)
    assert np.array_equal(got, -lc.astype(np.float64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_against_numpy_fp64_product(oracle, dtype):
    # a different implementation (BLAS) of the same definition
    M, N, K = 150, 130, 700
    la = pi.logical_matrix(61, 0, M, K, "normal", 1.0, dtype)
    lb = pi.logical_matrix(61, 1, K, N, "normal", 1.0, dtype)
    got = oracle.gemm(dtype, 0, 0, M, N, K, 1.0, la, lb)
    want = pi.to_f64(la, dtype) @ pi.to_f64(lb, dtype)
    assert oracle.rel_frobenius(got, want) < 1e-14
    # fp64 accumulation bound: |err| <= K * 2^-53 * sum |a||b|
    bound = K * 2.0 ** -53 * (np.abs(pi.to_f64(la, dtype)) @ np.abs(pi.to_f64(lb, dtype)))
    exact = np.array([[sum(map(float.__mul__, map(float, pi.to_f64(la, dtype)[i]), map(float, pi.to_f64(lb, dtype)[:, j])))
                       for j in range(3)] for i in range(3)])
    assert (np.abs(got[:3, :3] - exact) <= bound[:3, :3]).all()


def test_exact_rational_check_small(oracle):
    # exact arithmetic with Python fractions on a tiny fp32 case
    from fractions import Fraction
    M, N, K = 3, 4, 9
    la = pi.logical_matrix(71, 0, M, K, "uniform", 1.0, pi.F32)
    lb = pi.logical_matrix(71, 1, K, N, "uniform", 1.0, pi.F32)
    got = oracle.gemm(pi.F32, 0, 0, M, N, K, 1.0, la, lb)
    for i in range(M):
        for j in range(N):
            ex = sum(Fraction(float(la[i, k])) * Fraction(float(lb[k, j])) for k in range(K))
            assert abs(Fraction(float(got[i, j])) - ex) <= Fraction(K, 2 ** 53) * 9


def test_row_subset_matches_full(oracle):
    M, N, K = 40, 33, 50
    la = pi.logical_matrix(81, 0, M, K, "uniform", 1.0, pi.BF16)
    lb = pi.logical_matrix(81, 1, K, N, "uniform", 1.0, pi.BF16)
    lc = pi.logical_matrix(81, 2, M, N, "uniform", 1.0, pi.BF16)
    full = oracle.gemm(pi.BF16, 0, 1, M, N, K, 1.5, la, np.ascontiguousarray(lb.T), 0.5, lc)
    rows = [39, 0, 17, 17, 5]
    sub = oracle.gemm(pi.BF16, 0, 1, M, N, K, 1.5, la, np.ascontiguousarray(lb.T), 0.5, lc, rows=rows)
    assert np.array_equal(sub, full[rows])


def test_decoders_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want16 = bits.view(np.float16).astype(np.float64)
    wantbf = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    for b in range(65536):
        g16, gbf = oracle.decode_f16(b), oracle.decode_bf16(b)
        w16, wbf = want16[b], wantbf[b]
        assert (g16 == w16 and np.signbit(g16) == np.signbit(w16)) or (np.isnan(g16) and np.isnan(w16)), b
        assert (gbf == wbf and np.signbit(gbf) == np.signbit(wbf)) or (np.isnan(gbf) and np.isnan(wbf)), b


def test_rejects_bad_arguments(oracle):
    a = np.zeros((4, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.gemm(pi.F32, 0, 0, 4, 4, 5, 1.0, a, a)          # lda < K
    with pytest.raises(ValueError):
        oracle.gemm(pi.F32, 0, 0, 4, 4, 4, 1.0, a, a, rows=[4])  # row out of range
    with pytest.raises(ValueError):
        oracle.gemm(pi.F16, 0, 0, 4, 4, 4, 1.0, a, a)          # storage type mismatch


def test_rel_frobenius_measure(oracle):
    ref = np.array([[3.0, 4.0]])
    assert oracle.rel_frobenius(ref, ref) == 0.0
    assert abs(oracle.rel_frobenius(np.array([[3.0, 4.5]]), ref) - 0.1) < 1e-15
    assert oracle.rel_frobenius(np.array([[np.nan, 4.0]]), ref) == float("inf")
    assert oracle.rel_frobenius(np.zeros((1, 2)), np.zeros((1, 2))) == 0.0
    assert oracle.rel_frobenius(np.ones((1, 2)), np.zeros((1, 2))) == float("inf")


# ---------------------------------------------------------------------------
# The fused output step act(ref + bias)
# ---------------------------------------------------------------------------

def test_bias_act_hand_cases_fix_the_order_of_the_steps(oracle):
    # bias first, activation second: relu(-1 + 2) = 1, whereas relu(-1) + 2 = 2
    ref = np.array([[-1.0, 3.0], [-4.0, 0.5]])
    bias = np.array([2.0, -1.0], dtype=np.float32)
    out = oracle.bias_act(ref, 2, oracle.BIAS_PER_COLUMN, bias, oracle.ACT_RELU)
    assert out.tolist() == [[1.0, 2.0], [0.0, 0.0]]
    out = oracle.bias_act(ref, 2, oracle.BIAS_PER_ROW, bias, oracle.ACT_RELU)
    assert out.tolist() == [[1.0, 5.0], [0.0, 0.0]]
    # nothing asked for: unchanged, and the input is not written
    assert oracle.bias_act(ref, 2).tolist() == ref.tolist()
    assert ref.tolist() == [[-1.0, 3.0], [-4.0, 0.5]]


def test_bias_kinds_on_a_non_square_zero_product(oracle):
    # alpha = 0: the reference is all zero and the step leaves the broadcast bias behind
    M, N = 3, 5
    z = np.zeros((M, N))
    bc = np.arange(1, N + 1, dtype=np.float32)
    br = np.arange(10, 10 + M, dtype=np.float32)
    out = oracle.bias_act(z, M, oracle.BIAS_PER_COLUMN, bc)
    for i in range(M):
        assert out[i].tolist() == bc.tolist()
    out = oracle.bias_act(z, M, oracle.BIAS_PER_ROW, br)
    for j in range(N):
        assert out[:, j].tolist() == br.tolist()


def test_row_bias_follows_the_logical_row_of_a_subset(oracle):
    M, N = 6, 2
    br = np.arange(100, 100 + M, dtype=np.float32)
    rows = [4, 1, 5]
    out = oracle.bias_act(np.zeros((3, N)), M, oracle.BIAS_PER_ROW, br, rows=rows)
    assert out[:, 0].tolist() == [104.0, 101.0, 105.0]
    with pytest.raises(ValueError):
        oracle.bias_act(np.zeros((3, N)), M, oracle.BIAS_PER_ROW, br, rows=[0, 6, 1])


def test_relu_keeps_positives_and_clears_the_rest(oracle):
    x = np.array([[-2.5, -0.0, 0.0, 1e-300, 7.0, -1e-300]])
    out = oracle.bias_act(x, 1, act=oracle.ACT_RELU)
    assert out.tolist() == [[0.0, 0.0, 0.0, 1e-300, 7.0, 0.0]]


def test_gelu_tanh_against_torch_fp64_and_its_symmetry(oracle):
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 2, 500), np.linspace(-12, 12, 97), [0.0]]).reshape(1, -1)
    out = oracle.bias_act(x, 1, act=oracle.ACT_GELU_TANH)
    want = torch.nn.functional.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-300)
    # tanh is odd, so gelu(x) - gelu(-x) = x
    neg = oracle.bias_act(-x, 1, act=oracle.ACT_GELU_TANH)
    np.testing.assert_allclose(out - neg, x, rtol=1e-13, atol=1e-15)
    # far tails: identity on the right, zero on the left; and gelu(0) = 0
    tails = oracle.bias_act(np.array([[30.0, -30.0, 0.0]]), 1, act=oracle.ACT_GELU_TANH)
    assert tails.tolist() == [[30.0, 0.0, 0.0]]          # (-0.0 == 0.0)


def test_bias_act_composes_with_gemm_on_integers(oracle):
    # exact small-integer product, then bias and relu by hand
    M, N, K = 4, 3, 5
    rng = np.random.default_rng(11)
    a = rng.integers(-3, 4, (M, K)).astype(np.float32)
    b = rng.integers(-3, 4, (K, N)).astype(np.float32)
    bias = rng.integers(-5, 6, N).astype(np.float32)
    ref = oracle.gemm(oracle.F32, 0, 0, M, N, K, 2.0, a, b)
    out = oracle.bias_act(ref, M, oracle.BIAS_PER_COLUMN, bias, oracle.ACT_RELU)
    for i in range(M):
        for j in range(N):
            s = 2 * sum(int(a[i, k]) * int(b[k, j]) for k in range(K)) + int(bias[j])
            assert out[i, j] == max(s, 0)


def test_c_in_of_another_storage_type(oracle):
    """16-bit operands with an fp32 C_in: exact integers against the int64 brute force,
    and a C_in value that only fp32 can hold must arrive unrounded."""
    M, N, K = 5, 7, 9
    for dtype in (pi.F16, pi.BF16):
        A = pi.small_int_matrix(40, 0, M, K, -3, 3, dtype)
        B = pi.small_int_matrix(40, 1, K, N, -3, 3, dtype)
        Cin = pi.small_int_matrix(40, 2, M, N + 2, -9, 9, pi.F32)
        got = oracle.gemm(dtype, 0, 0, M, N, K, 2.0, A, B, -3.0, Cin, cdtype=pi.F32)
        want = _brute_int(0, 0, M, N, K, 2, _int_values(A, dtype).ravel(), K, _int_values(B, dtype).ravel(), N,
                          -3, Cin.astype(np.int64).ravel(), N + 2)
        assert np.array_equal(got, want.astype(np.float64))
        fine = np.full((M, N), 1.0 + 2.0 ** -20, dtype=np.float32)        # not representable in 16 bits
        got = oracle.gemm(dtype, 0, 0, M, N, K, 0.0, A, B, 1.0, fine, cdtype=pi.F32)
        assert np.array_equal(got, fine.astype(np.float64))
        with pytest.raises(ValueError):
            oracle.gemm(dtype, 0, 0, M, N, K, 1.0, A, B, 1.0, fine)       # storage check still on
