"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Integer-valued cases must match exactly; floating
point cases within the stated relative Frobenius error (1e-5 fp32, 2e-2 f16 and
bf16)."""
import itertools
import re

import numpy as np
import pytest

import peak_inputs as pi

pytestmark = pytest.mark.gpu

DTYPES = [pi.F32, pi.F16, pi.BF16]
LAYOUTS = list(itertools.product([0, 1], [0, 1]))


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from tests import gpu_util
    return gpu_util


def _stored(seed, dtype, M, N, K, transA, transB, pad=(0, 0, 0), ints=False, dist="uniform", scale=1.0, amp=2):
    if ints:
        la = pi.small_int_matrix(seed, 0, M, K, -amp, amp, dtype)
        lb = pi.small_int_matrix(seed, 1, K, N, -amp, amp, dtype)
        lc = pi.small_int_matrix(seed, 2, M, N, -3, 3, dtype)
    else:
        la = pi.logical_matrix(seed, 0, M, K, dist, scale, dtype)
        lb = pi.logical_matrix(seed, 1, K, N, dist, scale, dtype)
        lc = pi.logical_matrix(seed, 2, M, N, dist, 1.0, dtype)
    A = pi.store(la, bool(transA), (M if transA else K) + pad[0])
    B = pi.store(lb, bool(transB), (K if transB else N) + pad[1])
    C = pi.store(lc, False, N + pad[2])
    return A, B, C


def _skinny_max_m(name):
    """Largest M of a streaming variant: "_m<rows>n..." in the names that say it, else 16."""
    m = re.search(r"skinny_m(\d+)n", name)
    return int(m.group(1)) if m else 16


def _check_padding(raw, C0, M, N):
    # everything outside the logical M x N block must be byte-identical to before
    assert np.array_equal(raw[:, N:].view(np.uint8), C0[:, N:].view(np.uint8))
    assert np.array_equal(raw[M:, :].view(np.uint8), C0[M:, :].view(np.uint8))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_exact_integers_every_variant(gu, oracle, dtype, transA, transB):
    """Small integers: products and sums are exact in fp32, results (|c| <= 256)
    exact in every storage type, so the match must be bitwise.  Pins the MFMA
    fragment layout, the swizzle, the transposing stores and the edge masks of
    every kernel variant built for the layout."""
    for vid, name in gu.variants_for(dtype, transA, transB):
        direct = bool(re.search(r"_(?:d|t|p|pt|m)\d", name)) or "skinny" in name
        # K <= 64 keeps |sum| <= 4*64 = 256
        if "skinny" in name:
            m = re.search(r"k(\d+)s", name)
            ks = int(m.group(1)) if m else (64 if "skinnyreg" in name else 128)
            mm = _skinny_max_m(name)
            n2 = 130 if transB else 136                    # B as [k][n] rows: N a whole number of 16-byte chunks
            shapes = [(mm, 192, ks), (mm - 9, n2, 2 * ks), (1, 64, ks)] + ([(mm - 15, 72, ks)] if mm > 16 else [])
        elif direct:
            bk = 32 if ("f32" in name or "k32" in name) else 64
            epc = 16 // pi.DTYPE_SIZE[dtype]
            # the last two stop K inside a K tile, at a 16-byte chunk boundary
            shapes = [(256, 256, bk), (300, 504, 2 * bk if 2 * bk <= 64 else bk), (100, 72, bk),
                      (300, 504, bk + epc), (70, 40, bk - epc)]
            if transA:
                # A staged as [k][m] rows: M a whole number of 16-byte chunks
                shapes = [(-(-M // epc) * epc, N, K) for M, N, K in shapes]
                if not transB:
                    shapes.append((72, 40, bk + 5))        # both operands [k][.]: K may end anywhere
        else:
            shapes = [(128, 128, 64), (200, 333, 40), (77, 5, 33), (1, 1, 1), (129, 257, 64)]
        for case, (M, N, K) in enumerate(shapes):
            for alpha, beta in [(1.0, 0.0), (-1.0, 2.0)]:
                pad = (0, 0, 0) if direct else (case % 2 * 3, case % 2 * 5, case % 2 * 7)
                A, B, C = _stored(1000 + vid * 10 + case, dtype, M, N, K, transA, transB, pad, ints=True,
                                  amp=1 if K > 64 else 2)
                if direct:
                    # aligned leading dimensions for the direct kernels
                    al = 16 // pi.DTYPE_SIZE[dtype]
                    ok = A.shape[1] % al == 0 and B.shape[1] % al == 0
                    if not ok:
                        la = -(-A.shape[1] // al) * al
                        lb = -(-B.shape[1] // al) * al
                        A = np.pad(A, ((0, 0), (0, la - A.shape[1])))
                        B = np.pad(B, ((0, 0), (0, lb - B.shape[1])))
                C0 = C if beta != 0 else gu.nan_fill(C.shape[0], C.shape[1], dtype)
                ref = oracle.gemm(dtype, transA, transB, M, N, K, alpha, A, B, beta, C if beta != 0 else None)
                got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, alpha, beta, A, B, C0,
                                             flags=gu.pg.force_flags(variant=vid))
                assert np.array_equal(got, ref), (name, M, N, K, alpha, beta, info)
                _check_padding(raw, C0, M, N)


@pytest.mark.parametrize("dtype", DTYPES)
def test_random_every_direct_variant_deep_k(gu, oracle, dtype):
    """Forced direct-to-LDS and streaming variants over enough K tiles to wrap
    their staging rings several times, ragged M and N."""
    for transA, transB in LAYOUTS:
        for vid, name in gu.variants_for(dtype, transA, transB):
            if not (re.search(r"_(?:d|t|p|pt|m)\d", name) or "skinny" in name):
                continue
            # tiled kernels also get a K that ends inside the last K tile (of the last K slice)
            shapes = [(_skinny_max_m(name) - 3, 1000, 4096)] if "skinny" in name else [(300, 520, 1024), (260, 264, 1000)]
            if transA and "skinny" not in name:
                shapes = [(304, 520, 1024), (264, 264, 1000)] + ([(264, 264, 1003)] if not transB else [])
            for M, N, K in shapes:
                A, B, C = _stored(6000 + vid, dtype, M, N, K, transA, transB)
                ref, bound = gu.elementwise_bound(oracle, dtype, transA, transB, M, N, K, 1.0, A, B, 0.25, C)
                for split in (None, 3):
                    got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, 1.0, 0.25, A, B, C,
                                                 flags=gu.pg.force_flags(variant=vid, split=split))
                    err = oracle.rel_frobenius(got, ref)
                    assert err <= gu.TOL[dtype], (info, M, N, K, err)
                    gu.assert_elementwise(got, ref, bound, (info, M, N, K))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("transA,transB", LAYOUTS)
def test_random_against_oracle_auto_selection(gu, oracle, dtype, transA, transB):
    """Selector's own choice, sizes spanning several tiles with ragged tails."""
    for case, (M, N, K) in enumerate([(384, 320, 512), (513, 259, 1000), (33, 1100, 200), (700, 70, 4096)]):
        A, B, C = _stored(2000 + case, dtype, M, N, K, transA, transB)
        for alpha, beta in [(1.0, 0.0), (0.75, -0.5)]:
            C0 = C if beta != 0 else gu.nan_fill(M, N, dtype)
            got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, alpha, beta, A, B, C0)
            gu.check_against_oracle(oracle, got, dtype, transA, transB, M, N, K, alpha, A, B, beta, C,
                                    what=(info, M, N, K, alpha, beta))


@pytest.mark.parametrize("dtype", DTYPES)
def test_unaligned_operands_and_odd_leading_dimensions(gu, oracle, dtype):
    """Base pointers off 16-byte alignment and odd row strides force the element
    loaders and scalar stores."""
    M, N, K = 150, 97, 203
    for transA, transB in LAYOUTS:
        A, B, C = _stored(3000, dtype, M, N, K, transA, transB, pad=(1, 3, 1))
        es = pi.DTYPE_SIZE[dtype]
        # shift A and B by one element inside a larger allocation
        A1 = np.concatenate([A.ravel()[:1], A.ravel()]).reshape(1, -1)
        B1 = np.concatenate([B.ravel()[:1], B.ravel()]).reshape(1, -1)
        ref = oracle.gemm(dtype, transA, transB, M, N, K, 1.0, A, B, 0.5, C)
        dA, dB, dC = gu.to_dev(A1), gu.to_dev(B1), gu.to_dev(C)
        import torch
        with gu.pg.Plan(M, N, K, dtype, transA, transB, A.shape[1], B.shape[1], C.shape[1]) as plan:
            ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
            plan.run(1.0, dA.data_ptr() + es, dB.data_ptr() + es, 0.5, dC.data_ptr(), ws.data_ptr(),
                     plan.workspace_bytes, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            info = plan.info()
        raw = gu.from_dev(dC, dtype)
        got = pi.to_f64(np.ascontiguousarray(raw[:M, :N]), dtype)
        assert oracle.rel_frobenius(got, ref) <= gu.TOL[dtype], (info, transA, transB)
        gu.check_against_oracle(oracle, got, dtype, transA, transB, M, N, K, 1.0, A, B, 0.5, C, what=(info, transA, transB))
        _check_padding(raw, C, M, N)


@pytest.mark.parametrize("dtype", DTYPES)
def test_split_k_forced_and_deterministic(gu, oracle, dtype):
    M, N, K = 192, 160, 2048
    transA, transB = 0, 1
    A, B, C = _stored(4000, dtype, M, N, K, transA, transB)
    ref = oracle.gemm(dtype, transA, transB, M, N, K, 1.25, A, B, 0.5, C)
    outs = []
    for split in (1, 3, 8):
        got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, 1.25, 0.5, A, B, C,
                                     flags=gu.pg.force_flags(split=split))
        assert ("split=%d" % split) in info or split > 1, info
        assert oracle.rel_frobenius(got, ref) <= gu.TOL[dtype], info
        gu.check_against_oracle(oracle, got, dtype, transA, transB, M, N, K, 1.25, A, B, 0.5, C, what=info)
        again, raw2, _ = gu.run_gemm(dtype, transA, transB, M, N, K, 1.25, 0.5, A, B, C,
                                     flags=gu.pg.force_flags(split=split))
        assert np.array_equal(raw.view(np.uint8), raw2.view(np.uint8)), "run-to-run bits differ: " + info
        outs.append(got)


@pytest.mark.parametrize("dtype", DTYPES)
def test_degenerate_cases(gu, oracle, dtype):
    import torch
    M, N, K = 40, 24, 16
    A, B, C = _stored(5000, dtype, M, N, K, 0, 0, pad=(0, 0, 4))
    # alpha == 0: C = beta*C, operands not read (NULL pointers)
    with gu.pg.Plan(M, N, K, dtype, 0, 0, K, N, N + 4) as plan:
        dC = gu.to_dev(C)
        plan.run(0.0, 0, 0, -2.0, dC.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        raw = gu.from_dev(dC, dtype)
        assert np.array_equal(pi.to_f64(np.ascontiguousarray(raw[:, :N]), dtype), -2.0 * pi.to_f64(np.ascontiguousarray(C[:, :N]), dtype))
        _check_padding(raw, C, M, N)
    # K == 0 with beta == 0: zeros, NaN in C_in not propagated
    with gu.pg.Plan(M, N, 0, dtype, 0, 0, 1, N, N + 4) as plan:
        C0 = gu.nan_fill(M, N + 4, dtype)
        dC = gu.to_dev(C0)
        plan.run(1.0, 0, 0, 0.0, dC.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        raw = gu.from_dev(dC, dtype)
        assert (pi.to_f64(np.ascontiguousarray(raw[:, :N]), dtype) == 0).all()
        _check_padding(raw, C0, M, N)
    # M == 0 / N == 0: nothing happens
    with gu.pg.Plan(0, N, K, dtype) as plan:
        plan.run(1.0, 0, 0, 0.0, 0)
    with gu.pg.Plan(M, 0, K, dtype) as plan:
        plan.run(1.0, 0, 0, 0.0, 0)
    # identity and permutation, exact
    Kp = 96
    la = pi.logical_matrix(5001, 0, 70, Kp, "uniform", 1.0, dtype)
    perm = np.random.default_rng(9).permutation(Kp)
    P = np.zeros((Kp, Kp), np.float32)
    P[perm, np.arange(Kp)] = 1.0
    Pst = pi.round_to_dtype(P, dtype).reshape(Kp, Kp)
    got, _, info = gu.run_gemm(dtype, 0, 0, 70, Kp, Kp, 1.0, 0.0, la, Pst, gu.nan_fill(70, Kp, dtype))
    assert np.array_equal(got, pi.to_f64(la, dtype)[:, perm]), info


def test_error_paths_on_device(gu):
    import torch
    pg = gu.pg
    M, N, K = 64, 64, 4096
    with pg.Plan(M, N, K, pg.PEAK_DT_BF16, 0, 1, flags=pg.force_flags(split=4)) as plan:
        assert plan.workspace_bytes == 4 * M * N * 4
        a = torch.zeros(M * K, dtype=torch.int16, device="cuda")
        c = torch.zeros(M * N, dtype=torch.int16, device="cuda")
        st = pg.peak_gemm_run(plan.handle, 1.0, a.data_ptr(), a.data_ptr(), 0.0, c.data_ptr(), 0, 0, 0)
        assert st == pg.PEAK_ERR_WORKSPACE
        ws = torch.zeros(1024, dtype=torch.uint8, device="cuda")
        st = pg.peak_gemm_run(plan.handle, 1.0, a.data_ptr(), a.data_ptr(), 0.0, c.data_ptr(), ws.data_ptr(), 1024, 0)
        assert st == pg.PEAK_ERR_WORKSPACE
        st = pg.peak_gemm_run(plan.handle, 1.0, 0, a.data_ptr(), 0.0, c.data_ptr(), 0, 0, 0)
        assert st == pg.PEAK_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", [pi.F16, pi.BF16])
def test_two_workgroups_per_cu_with_assembly_issued_reads(gu, oracle, dtype):
    """128x128 tiles take 64 KB of LDS, so a grid beyond 256 workgroups puts two on
    a CU.  The kernels that stage an operand as [k][.] rows issue their transposing
    LDS reads as assembly; the last ones of the K loop feed nothing, and must still
    have returned before the epilogue reuses their registers (a late return once
    overwrote a lane index there).  Full result against the oracle on sampled rows."""
    M, N, K = 2560, 2560, 256
    pre = "f16" if dtype == pi.F16 else "bf16"
    names = [gu.pg.peak_gemm_variant_name(i) for i in range(gu.pg.peak_gemm_variant_count())]
    rows = sorted({0, 1, 127, 128, 1279, 2431, 2559} | set(range(640, 648)))
    for suffix, tA, tB in [("t128x128w4_nn", 0, 0), ("t128x128w4_tn", 1, 0), ("t128x128w4_tt", 1, 1)]:
        vid = names.index("%s_%s" % (pre, suffix))
        A, B, C = _stored(9100 + vid, dtype, M, N, K, tA, tB, scale=0.25)
        ref = oracle.gemm(dtype, tA, tB, M, N, K, 1.0, A, B, 0.0, None, rows=rows)
        C0 = gu.nan_fill(M, N, dtype)
        for rep in range(3):
            got, raw, info = gu.run_gemm(dtype, tA, tB, M, N, K, 1.0, 0.0, A, B, C0, flags=gu.pg.force_flags(variant=vid))
            assert "grid=400" in info, info
            err = oracle.rel_frobenius(got[rows], ref)
            assert err <= gu.TOL[dtype], (info, rep, err)
            assert np.isfinite(got).all(), info
            if rep == 0:
                gu.check_against_oracle(oracle, got, dtype, tA, tB, M, N, K, 1.0, A, B, 0.0, None, rows=rows, what=info)


@pytest.mark.parametrize("dtype", DTYPES)
def test_more_tiles_than_workgroups(gu, oracle, dtype):
    """More tiles than the chip has CUs (and not a multiple of it), for the kernels that
    hold a CU alone: every CU gets several workgroups one after another and the last
    round is partial.  Exact integers, checked on sampled rows including the first and
    last tile rows."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    M, N, K = 4352 + 40, 4352 + 8, 128                       # 18 x 18 tiles of 256 x 256
    rows = sorted({0, 1, 255, 256, 2047, 2048, 4351, 4352, M - 1} | {int(x) for x in np.random.default_rng(1).integers(0, M, 16)})
    for transA, transB in [(0, 1), (0, 0), (1, 0)]:
        ran = 0
        A, B, C = _stored(9000 + transA * 2 + transB, dtype, M, N, K, transA, transB, ints=True, amp=1)
        ref = oracle.gemm(dtype, transA, transB, M, N, K, 1.0, A, B, 2.0, C, rows=rows)
        for vid, name in gu.variants_for(dtype, transA, transB):
            try:
                with gu.pg.Plan(M, N, K, dtype, transA, transB, flags=gu.pg.force_flags(variant=vid, split=1)) as plan:
                    info = plan.info()
            except gu.pg.PeakError as e:
                assert e.status == gu.pg.PEAK_ERR_UNSUPPORTED
                continue
            lds = int(re.search(r"lds=(\d+)", info).group(1))
            grid = int(re.search(r"grid=(\d+)", info).group(1))
            if "skinny" in name or lds <= 80 * 1024:
                continue
            assert grid > cus, info
            got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, 1.0, 2.0, A, B, C,
                                         flags=gu.pg.force_flags(variant=vid, split=1))
            assert np.array_equal(got[rows], ref), (name, info)
            ran += 1
        assert ran >= 1, (dtype, transA, transB)


@pytest.mark.parametrize("dtype", DTYPES)
def test_exact_integers_deep_k_every_direct_variant(gu, oracle, dtype):
    """Entries in {-1, 0, 1} over 16 and more K tiles, so every staging ring wraps
    several times in its steady state: all sums are exact in fp32, so a stale stage,
    a fragment read before its load has landed or a slice boundary off by one shows
    as a wrong integer.  Every direct-to-LDS and streaming variant, split and unsplit,
    K ending inside a K tile as well.  16-bit kernels are checked twice: with C in
    their own storage type (the sums stay within the integers it holds exactly,
    asserted) and with fp32 C (PEAK_GEMM_C_F32), which takes the other readout."""
    limit = {pi.F32: 2 ** 24, pi.F16: 2048, pi.BF16: 256}[dtype]
    for transA, transB in LAYOUTS:
        for vid, name in gu.variants_for(dtype, transA, transB):
            if not (re.search(r"_(?:d|t|p|pt|m)\d", name) or "skinny" in name):
                continue
            if "skinny" in name:
                mm = _skinny_max_m(name)
                shapes = [(mm - 3, 1000, 4096), (mm, 264, 4096)]
            elif transA:
                shapes = [(304, 520, 1024), (264, 264, 2056 if transB else 2051)]
            else:
                shapes = [(300, 520, 1024), (260, 264, 2056)]
            if "skinny" not in name:
                # one row of tiles, several columns: the plans that start each workgroup at another K tile
                shapes.append((104, 520, 2056 if transB or not transA else 2051))
            for case, (M, N, K) in enumerate(shapes):
                A, B, C = _stored(7000 + vid * 4 + case, dtype, M, N, K, transA, transB, ints=True, amp=1)
                ref = oracle.gemm(dtype, transA, transB, M, N, K, 1.0, A, B, 1.0, C)
                assert np.abs(ref).max() <= limit, (name, np.abs(ref).max())
                for split in (None, 3):
                    got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, 1.0, 1.0, A, B, C,
                                                 flags=gu.pg.force_flags(variant=vid, split=split))
                    assert np.array_equal(got, ref), (info, M, N, K, int((got != ref).sum()))
                    if dtype != pi.F32 and split is None:
                        C32 = pi.to_f64(C, dtype).astype(np.float32)
                        got, raw, info = gu.run_gemm(dtype, transA, transB, M, N, K, 1.0, 1.0, A, B, C32,
                                                     flags=gu.pg.force_flags(variant=vid), cdtype=pi.F32)
                        assert np.array_equal(got, ref), (info, "fp32 C", M, N, K, int((got != ref).sum()))


@pytest.mark.parametrize("dtype", DTYPES)
def test_operand_base_off_16_bytes_with_aligned_rows(gu, oracle, dtype):
    """Leading dimensions that suit the 16-byte copies, but A or B starting one
    element into an allocation (a view into a larger matrix): legal by the interface,
    which asks for element alignment only.  The plan is made without the addresses, so
    it holds a direct-to-LDS variant; the run must fall back to the plan's
    register-staged stand-in and still match the oracle, with and without a K split."""
    import torch
    es = pi.DTYPE_SIZE[dtype]
    for transA, transB in LAYOUTS:
        for M, N, K, split in [(264, 520, 1024, None), (264, 520, 2048, 4), (16, 512, 1024, None)]:
            if M == 16 and (transA or not transB):
                continue                                   # the streaming kernels: both operands along K
            A, B, C = _stored(3100 + M, dtype, M, N, K, transA, transB)
            with gu.pg.Plan(M, N, K, dtype, transA, transB, flags=gu.pg.force_flags(split=split)) as plan:
                info = plan.info()
                assert re.search(r"variant=\d+:\w+_(?:d|t|m)\d|skinny", info), info      # a variant with alignment needs
                assert "unaligned=same" not in info, info
                ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
                for off_a, off_b in [(1, 0), (0, 1), (1, 1)]:
                    # the same values, one element into a larger allocation
                    A1 = np.concatenate([A.ravel()[:1], A.ravel()]).reshape(1, -1)
                    B1 = np.concatenate([B.ravel()[:1], B.ravel()]).reshape(1, -1)
                    dA, dB, dC = gu.to_dev(A1 if off_a else A), gu.to_dev(B1 if off_b else B), gu.to_dev(C)
                    plan.run(0.5, dA.data_ptr() + off_a * es, dB.data_ptr() + off_b * es, 2.0, dC.data_ptr(),
                             ws.data_ptr(), plan.workspace_bytes, torch.cuda.current_stream().cuda_stream)
                    torch.cuda.synchronize()
                    raw = gu.from_dev(dC, dtype)
                    got = pi.to_f64(np.ascontiguousarray(raw[:M, :N]), dtype)
                    gu.check_against_oracle(oracle, got, dtype, transA, transB, M, N, K, 0.5, A, B, 2.0, C,
                                            what=(info, transA, transB, off_a, off_b))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("transB", [0, 1])
def test_streaming_variants_with_a_stored_k_by_m(gu, oracle, dtype, transB):
    """Every streaming variant on an A stored K x M: the run first writes A out along K
    into the workspace (behind the Split-K partials) and the kernel reads that copy.
    Exact integers over many K tiles, split and unsplit, odd leading dimension of A (the
    copy is aligned whatever A's rows are), A's base one element into its allocation, a K
    that is not a whole number of 64-row blocks of the transposition; then random data
    against the per-element bound.  Padding of C must stay untouched."""
    limit = {pi.F32: 2 ** 24, pi.F16: 2048, pi.BF16: 256}[dtype]
    es = pi.DTYPE_SIZE[dtype]
    for vid, name in gu.variants_for(dtype, 0, transB):
        if "skinny" not in name or "skinnyreg" in name:
            continue
        m = re.search(r"k(\d+)s", name)
        ks = int(m.group(1)) if m else 128
        mm = _skinny_max_m(name)
        n2 = 1000 if transB else 1032                       # B as [k][n] rows: N a whole number of 16-byte chunks
        for case, (M, N, K, pad_a, a_off) in enumerate([(mm, 264, min(16 * ks, 4096), 0, 0), (mm - 3, n2, 4096 + ks, 3, 0),
                                                        (1, 264, 8 * ks, 5, 1)]):
            A, B, C = _stored(9000 + vid * 4 + case, dtype, M, N, K, 1, transB, pad=(pad_a, 0, 7), ints=True, amp=1)
            ref = oracle.gemm(dtype, 1, transB, M, N, K, 1.0, A, B, 1.0, C)
            assert np.abs(ref).max() <= limit
            # a base one element in: the same values, shifted by one element in a longer allocation
            Adev = A if not a_off else np.concatenate([np.zeros(1, A.dtype), A.reshape(-1)]).reshape(1, -1)
            for split in (None, 3):
                if a_off:
                    # run_gemm takes the leading dimension from the array's row length: hand it the flat copy by hand
                    import torch
                    dA, dB, dC = gu.to_dev(Adev), gu.to_dev(B), gu.to_dev(C)
                    with gu.pg.Plan(M, N, K, dtype, 1, transB, A.shape[1], B.shape[1], C.shape[1],
                                    gu.pg.force_flags(variant=vid, split=split)) as plan:
                        info = plan.info()
                        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
                        plan.run(1.0, dA.data_ptr() + es, dB.data_ptr(), 1.0, dC.data_ptr(), ws.data_ptr(),
                                 plan.workspace_bytes, torch.cuda.current_stream().cuda_stream)
                        torch.cuda.synchronize()
                    raw = gu.from_dev(dC, dtype)
                    got = pi.to_f64(np.ascontiguousarray(raw[:M, :N]), dtype)
                else:
                    got, raw, info = gu.run_gemm(dtype, 1, transB, M, N, K, 1.0, 1.0, A, B, C,
                                                 flags=gu.pg.force_flags(variant=vid, split=split))
                assert name in info and info.endswith("acopy=1"), info
                assert np.array_equal(got, ref), (info, M, N, K, int((got != ref).sum()))
                _check_padding(raw, C, M, N)
        M, N, K = mm - 5 if mm > 16 else 13, n2, 2048
        A, B, C = _stored(9500 + vid, dtype, M, N, K, 1, transB, pad=(1, 0, 0))
        got, raw, info = gu.run_gemm(dtype, 1, transB, M, N, K, 0.5, -0.75, A, B, C, flags=gu.pg.force_flags(variant=vid))
        assert info.endswith("acopy=1"), info
        gu.check_against_oracle(oracle, got, dtype, 1, transB, M, N, K, 0.5, A, B, -0.75, C, what=(info, M, N, K))
    # the selector's own plan for a streamed operand of some MB, and the workspace check of the run
    M, N, K = 24, 4104 if transB else 4096, 2048
    A, B, C = _stored(9900, dtype, M, N, K, 1, transB)
    got, raw, info = gu.run_gemm(dtype, 1, transB, M, N, K, 1.0, 0.0, A, B, gu.nan_fill(M, N, dtype))
    assert "skinny" in info and info.endswith("acopy=1"), info
    gu.check_against_oracle(oracle, got, dtype, 1, transB, M, N, K, 1.0, A, B, 0.0, C, what=(info, M, N, K))
    # B one element into its allocation: the run takes the plan's register-staged stand-in, which reads A as it lies
    Bflat = np.concatenate([np.zeros(1, B.dtype), B.reshape(-1)]).reshape(1, -1)
    import torch
    dA, dB, dC = gu.to_dev(A), gu.to_dev(Bflat), gu.to_dev(gu.nan_fill(M, N, dtype))
    with gu.pg.Plan(M, N, K, dtype, 1, transB, A.shape[1], B.shape[1], N) as plan:
        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
        plan.run(1.0, dA.data_ptr(), dB.data_ptr() + es, 0.0, dC.data_ptr(), ws.data_ptr(), plan.workspace_bytes,
                 torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        info2 = plan.info()
    got = pi.to_f64(np.ascontiguousarray(gu.from_dev(dC, dtype)[:M, :N]), dtype)
    gu.check_against_oracle(oracle, got, dtype, 1, transB, M, N, K, 1.0, A, B, 0.0, C, what=(info2, "B base off 16 bytes"))
    with gu.pg.Plan(M, N, K, dtype, 1, transB) as plan:
        assert plan.workspace_bytes >= M * K * es
        dA, dB, dC = gu.to_dev(A), gu.to_dev(B), gu.to_dev(C)
        with pytest.raises(gu.pg.PeakError) as e:
            plan.run(1.0, dA.data_ptr(), dB.data_ptr(), 0.0, dC.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
        assert e.value.status == gu.pg.PEAK_ERR_WORKSPACE
