"""Host side of the C ABI, no GPU needed: the library loads, exports every
symbol the header declares, validates descriptors and plans the graded
workloads sensibly.  No compute call is made here."""
import ctypes
import os
import re

import pytest

import paper_2512_19018_amd as pg
import peak_inputs as pi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(M=64, N=64, K=64, dtype=pg.PEAK_DT_BF16, tA=0, tB=0, lda=None, ldb=None, ldc=None, flags=0):
    lda = lda if lda is not None else (M if tA else K)
    ldb = ldb if ldb is not None else (K if tB else N)
    ldc = ldc if ldc is not None else N
    return pg.PeakGemmDesc(M, N, K, lda, ldb, ldc, tA, tB, dtype, flags)


def test_every_declared_symbol_is_exported():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert len(headers) >= 2
    header = "\n".join(open(h).read() for h in headers)
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(peak_[a-z_]+)\s*\(", header))
    assert {"peak_calib_mfma", "peak_calib_read", "peak_calib_lds_load"} <= names
    assert {"peak_gemm_create", "peak_gemm_run", "peak_gemm_destroy", "peak_gemm_workspace_bytes",
            "peak_status_string", "peak_gemm_plan_info"} <= names
    lib = pg.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    seen = set()
    for s in range(6):
        txt = pg.peak_status_string(s)
        assert txt and txt not in seen
        seen.add(txt)
    assert pg.peak_status_string(99)


@pytest.mark.parametrize("bad", [
    dict(M=-1), dict(N=-5), dict(K=-2), dict(dtype=7), dict(tA=2), dict(tB=-1),
    dict(lda=63), dict(ldb=10), dict(ldc=1), dict(tA=1, lda=63), dict(tB=1, ldb=63), dict(flags=1 << 20),
])
def test_create_rejects_bad_descriptors(bad):
    st, h = pg.peak_gemm_create(_desc(**bad))
    assert st == pg.PEAK_ERR_INVALID_ARG and h is None


def test_create_null_pointers():
    lib = pg.load_library()
    h = ctypes.c_void_p(1234)
    assert lib.peak_gemm_create(None, ctypes.byref(h)) == pg.PEAK_ERR_INVALID_ARG
    assert h.value is None                      # *out_plan is cleared on error
    d = _desc()
    assert lib.peak_gemm_create(ctypes.byref(d), None) == pg.PEAK_ERR_INVALID_ARG
    assert lib.peak_gemm_destroy(None) == pg.PEAK_OK
    assert lib.peak_gemm_workspace_bytes(None) == 0
    assert lib.peak_gemm_run(None, 1.0, None, None, 0.0, None, None, 0, None) == pg.PEAK_ERR_INVALID_ARG


def test_degenerate_sizes_make_plans():
    for kw in (dict(M=0), dict(N=0, ldb=1, ldc=1), dict(K=0, lda=1, ldb=64)):
        st, h = pg.peak_gemm_create(_desc(**kw))
        assert st == pg.PEAK_OK
        assert pg.peak_gemm_workspace_bytes(h) == 0
        assert "degenerate" in pg.peak_gemm_plan_info(h)
        pg.peak_gemm_destroy(h)


def test_forced_variant_must_fit():
    names = [pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())]
    assert pg.peak_gemm_variant_name(-1) is None and pg.peak_gemm_variant_name(len(names)) is None
    f32_nn = names.index("f32_r128x128_nn")
    # wrong dtype, wrong layout: the invalid-configuration sentinel, not a crash
    st, _ = pg.peak_gemm_create(_desc(dtype=pg.PEAK_DT_BF16, flags=pg.force_flags(variant=f32_nn)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    st, _ = pg.peak_gemm_create(_desc(dtype=pg.PEAK_DT_F32, tB=1, flags=pg.force_flags(variant=f32_nn)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    st, h = pg.peak_gemm_create(_desc(dtype=pg.PEAK_DT_F32, flags=pg.force_flags(variant=f32_nn)))
    assert st == pg.PEAK_OK and "f32_r128x128_nn" in pg.peak_gemm_plan_info(h)
    pg.peak_gemm_destroy(h)
    # direct-to-LDS variants need K a whole number of 16-byte chunks and 16-byte aligned rows
    direct = names.index("bf16_d256x256w8_nt")
    st, _ = pg.peak_gemm_create(_desc(512, 512, 1004, tB=1, lda=1008, ldb=1008, flags=pg.force_flags(variant=direct)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    st, h = pg.peak_gemm_create(_desc(512, 512, 1000, tB=1, flags=pg.force_flags(variant=direct)))
    assert st == pg.PEAK_OK
    pg.peak_gemm_destroy(h)
    # the streaming kernels for M <= 16 take whole K steps only
    skinny = names.index("bf16_skinny64k512s2_nt")
    st, _ = pg.peak_gemm_create(_desc(16, 512, 1000, tB=1, flags=pg.force_flags(variant=skinny)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    # [k][n] staging of B needs N a whole number of chunks as well
    tr = names.index("bf16_t256x256w8_nn")
    st, _ = pg.peak_gemm_create(_desc(512, 500, 1024, ldb=504, flags=pg.force_flags(variant=tr)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    st, _ = pg.peak_gemm_create(_desc(512, 512, 1024, tB=1, lda=1028, flags=pg.force_flags(variant=direct)))
    assert st == pg.PEAK_ERR_UNSUPPORTED
    st, h = pg.peak_gemm_create(_desc(512, 512, 1024, tB=1, flags=pg.force_flags(variant=direct)))
    assert st == pg.PEAK_OK
    pg.peak_gemm_destroy(h)
    st, _ = pg.peak_gemm_create(_desc(flags=pg.force_flags(variant=250)))
    assert st == pg.PEAK_ERR_UNSUPPORTED


def test_forced_split_and_workspace():
    with pg.Plan(100, 200, 4096, pg.PEAK_DT_F16, 0, 1, flags=pg.force_flags(split=4)) as p:
        assert "split=4" in p.info()
        assert p.workspace_bytes == 4 * 100 * 200 * 4
    with pg.Plan(100, 200, 64, pg.PEAK_DT_F16, 0, 1, flags=pg.force_flags(split=200)) as p:
        assert "split=1" in p.info() and p.workspace_bytes == 0     # never more slices than K tiles


def test_plans_for_the_graded_workloads():
    w = pi.WORKLOADS
    info = {}
    for name in ("C1", "C2", "C3", "C3b", "C4", "C5"):
        x = w[name]
        lda, ldb, ldc = x.ld()
        with pg.Plan(x.M, x.N, x.K, x.dtype, x.transA, x.transB, lda, ldb, ldc) as p:
            info[name] = p.info()
    assert "f32_" in info["C1"] and "_nn" in info["C1"]
    assert ("f32_d" in info["C2"] or "f32_t" in info["C2"]) and "_nn" in info["C2"]
    assert "bf16_m256x256" in info["C3"] and "_nt" in info["C3"] and "tiles 32x32" in info["C3"]
    assert "bf16_m256x256" in info["C3b"]
    assert "f16_m256x256" in info["C4"] and "_nn" in info["C4"] and "tiles 20x12" in info["C4"]
    assert "skinny" in info["C5"]


def test_every_layout_and_dtype_has_a_general_variant():
    # any alignment, any K: one of the register-staged kernels must accept it
    for dt in (pg.PEAK_DT_F32, pg.PEAK_DT_F16, pg.PEAK_DT_BF16):
        for tA in (0, 1):
            for tB in (0, 1):
                with pg.Plan(37, 53, 29, dt, tA, tB, (37 if tA else 29) + 1, (29 if tB else 53) + 3, 53 + 1) as p:
                    assert "_r" in p.info()


def test_too_large_dimensions_are_unsupported_not_fatal():
    st, _ = pg.peak_gemm_create(_desc(M=1 << 31, lda=64))
    assert st == pg.PEAK_ERR_UNSUPPORTED


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import importlib
    import paper_2512_19018_amd.binding as b
    monkeypatch.setenv("PEAK_GEMM_LIB", str(tmp_path / "nope.so"))
    monkeypatch.setattr(b, "_LIB", None)
    with pytest.raises(ImportError):
        b.load_library()
    monkeypatch.undo()
    importlib.reload(b)


def test_selector_table_overrides_the_cost_model(tmp_path):
    """A table from an offline sweep decides for the shapes it lists, if the
    variant fits; everything else goes through the cost model as before."""
    try:
        with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1) as p:
            default = p.info()
        assert "bf16_m256x256w" in default
        table = tmp_path / "table.txt"
        table.write_text("# comment\n"
                         "bf16 0 1 8192 8192 8192 bf16_d256x128w8_nt 2   # 900.0 us\n"
                         "\n"
                         "f32 0 0 4096 4096 4096 f32_t256x128w8_nn 1\n")
        assert pg.peak_gemm_load_tuning(str(table)) == 2
        with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1) as p:
            assert "bf16_d256x128w8_nt" in p.info() and "split=2" in p.info()
        with pg.Plan(4096, 4096, 4096, pg.PEAK_DT_F32, 0, 0) as p:
            assert "f32_t256x128w8_nn" in p.info()
        # same shape, but rows not 16-byte aligned: the tabled variant does not fit, the cost model decides
        with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1, lda=8193) as p:
            assert "bf16_r128x128_nt" in p.info()
        # another shape: untouched
        with pg.Plan(4096, 4096, 4096, pg.PEAK_DT_BF16, 0, 1) as p:
            assert "bf16_m256x256w" in p.info()
        # forcing still wins over the table
        names = [pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())]
        with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1,
                     flags=pg.force_flags(variant=names.index("bf16_d128x128w4_nt"))) as p:
            assert "bf16_d128x128w4_nt" in p.info()
        # a malformed file is refused and the table in force stays
        bad = tmp_path / "bad.txt"
        bad.write_text("bf16 0 1 8192 8192 8192 no_such_variant 1\n")
        assert pg.peak_gemm_load_tuning(str(bad)) == -1
        bad.write_text("bf16 0 1 8192 8192 8192 f32_t256x128w8_nn 1\n")      # dtype of the variant differs
        assert pg.peak_gemm_load_tuning(str(bad)) == -1
        assert pg.peak_gemm_load_tuning(str(tmp_path / "missing.txt")) == -1
        with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1) as p:
            assert "bf16_d256x128w8_nt" in p.info()
    finally:
        assert pg.peak_gemm_load_tuning(None) == 0
    with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1) as p:
        assert p.info() == default


def test_tuner_enumerates_only_accepted_settings():
    from paper_2512_19018_amd import tune
    cands = tune.candidates(pg.PEAK_DT_BF16, 0, 1, 256, 512, 1024)
    names = {c[1] for c in cands}
    assert "bf16_d256x256w8_nt" in names and "bf16_r128x128_nt" in names
    assert not any(n.startswith(("f16_", "f32_")) or n.endswith(("_nn", "_tt", "_tn")) for n in names)
    assert not any("skinny" in n for n in names)                   # M > 16
    assert len({(c[0], c[2]) for c in cands}) == len(cands)        # each (variant, effective split) once
    # the library's own choice wins ties within the margin, a clearly faster setting does not lose to it
    res = [(10.0, "a", 1), (10.1, "b", 2), (12.0, "c", 1)]
    assert tune.pick(res, ("b", 2), 0.015) == (10.1, "b", 2)
    assert tune.pick(res, ("c", 1), 0.015) == (10.0, "a", 1)
    assert tune.pick(res, ("zz", 1), 0.015) == (10.0, "a", 1)
    own = tune.own_choice(pg.PEAK_DT_BF16, 0, 1, 8192, 8192, 8192)
    assert own == ("bf16_m256x256w4a3_nt", 1)
    assert tune.is_streamk("variant=1:x split=4 grid=8 streamk=64 rot=0,0") and not tune.is_streamk("split=1 streamk=0 rot=0,0")
    line = tune.table_line(pg.PEAK_DT_BF16, 0, 1, 256, 512, 1024, "bf16_d256x256w8_nt", 4, 12.5)
    assert line.split()[:8] == ["bf16", "0", "1", "256", "512", "1024", "bf16_d256x256w8_nt", "4"]


def test_fused_run_checks_its_epilogue_before_anything_else():
    # no device is touched: the epilogue is validated first, and M == 0 launches nothing
    with pg.Plan(0, 8, 8, pg.PEAK_DT_F32) as plan:
        assert pg.peak_gemm_run_fused(plan.handle, 1.0, 0, 0, 0.0, 0, None) == pg.PEAK_OK
        ok = pg.PeakGemmEpilogue(None, pg.PEAK_BIAS_NONE, pg.PEAK_ACT_GELU_TANH)
        assert pg.peak_gemm_run_fused(plan.handle, 1.0, 0, 0, 0.0, 0, ok) == pg.PEAK_OK
        for bad in (pg.PeakGemmEpilogue(None, pg.PEAK_BIAS_PER_COLUMN, 0),      # bias missing
                    pg.PeakGemmEpilogue(0x1002, pg.PEAK_BIAS_PER_ROW, 0),       # bias not 4-byte aligned
                    pg.PeakGemmEpilogue(None, 3, 0), pg.PeakGemmEpilogue(None, -1, 0),
                    pg.PeakGemmEpilogue(None, 0, 3), pg.PeakGemmEpilogue(None, 0, -1)):
            assert pg.peak_gemm_run_fused(plan.handle, 1.0, 0, 0, 0.0, 0, bad) == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_gemm_run_fused(None, 1.0, 0, 0, 0.0, 0, None) == pg.PEAK_ERR_INVALID_ARG


def test_validator_sampling_is_seeded_and_keeps_a_plain_reference():
    from paper_2512_19018_amd import validate as val
    from paper_2512_19018_amd.tune import candidates
    cands = candidates(pg.PEAK_DT_BF16, 0, 1, 300, 520, 1000)
    assert len(cands) > 20
    assert val.sample_settings(cands, None) == cands and val.sample_settings(cands, 10 ** 6) == cands
    a, b = val.sample_settings(cands, 7, seed=1), val.sample_settings(cands, 7, seed=1)
    assert a == b and len(a) == 7 and len(set(a)) == 7 and all(x in cands for x in a)
    assert val.sample_settings(cands, 7, seed=2) != a
    ref = val.reference_setting(cands)
    assert "_r64x64_" in ref[1] and ref[2] == 1


def test_validator_guard_bands_notice_a_stray_write():
    # on host tensors: the check itself, with the mistake planted by the test
    import torch
    from paper_2512_19018_amd import validate as val
    for tdt, dt in ((torch.float32, pg.PEAK_DT_F32), (torch.bfloat16, pg.PEAK_DT_BF16), (torch.float16, pg.PEAK_DT_F16)):
        g = val._Guarded(torch, 3, 5, tdt, dt, torch.ones(3, 5, dtype=tdt), device="cpu")
        assert g.guards_intact()
        assert bool(torch.isnan(g.buf[:g.g].float()).all()) and bool(torch.isnan(g.buf[g.g + g.n:].float()).all())
        g.body.fill_(2.0)                         # inside: allowed
        assert g.guards_intact()
        g.buf[g.g + g.n] = 1.0                    # first element after the body
        assert not g.guards_intact()
        g = val._Guarded(torch, 3, 5, tdt, dt, None, device="cpu")
        assert bool(torch.isnan(g.body.float()).all())     # unfilled body is poisoned too
        g.buf[g.g - 1] = 0.0                      # last element before the body
        assert not g.guards_intact()


def test_fp32_c_flag_is_accepted_and_other_high_bits_are_not():
    st, h = pg.peak_gemm_create(_desc(flags=pg.PEAK_GEMM_C_F32))
    assert st == pg.PEAK_OK
    pg.peak_gemm_destroy(h)
    st, h = pg.peak_gemm_create(_desc(dtype=pg.PEAK_DT_F32, flags=pg.PEAK_GEMM_C_F32))
    assert st == pg.PEAK_OK
    pg.peak_gemm_destroy(h)
    for bad in (0x80000, 0x80000000, pg.PEAK_GEMM_C_F32 | 0x100000, pg.PEAK_GEMM_STREAMK_ON | pg.PEAK_GEMM_STREAMK_OFF):
        st, h = pg.peak_gemm_create(_desc(flags=bad))
        assert st == pg.PEAK_ERR_INVALID_ARG and h is None
    assert pg.force_flags(3, 2, c_f32=True) == (4 | (2 << 8) | pg.PEAK_GEMM_C_F32)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def _plan_info_in_fresh_process(env_extra, shape):
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r); import paper_2512_19018_amd as pg\n"
            "with pg.Plan(%d, %d, %d, pg.PEAK_DT_BF16, 0, 1) as p: print(p.info())" % ((ROOT,) + shape))
    env = dict(os.environ)
    env.pop("PEAK_GEMM_TUNING", None)
    env.update(env_extra)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 0, r.stderr
    return r.stdout.strip()


def test_shipped_selector_table_is_loaded_by_default():
    """The table beside the shared object decides for the shapes it lists from the
    first create on; PEAK_GEMM_TUNING names another table or, empty, turns tables off."""
    table = os.path.join(ROOT, "paper_2512_19018_amd", "peak_gemm_tuning.txt")
    rows = [l.split("#")[0].split() for l in open(table) if l.split("#")[0].strip()]
    assert len(rows) >= 40 and all(len(r) == 8 for r in rows)
    names = {pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())}
    assert all(r[6] in names for r in rows)
    # a small problem the cost model is known to rank badly
    row = [r for r in rows if r[:6] == ["bf16", "0", "1", "256", "256", "1024"]][0]
    with_table = _plan_info_in_fresh_process({}, (256, 256, 1024))
    assert row[6] in with_table and "split=%s " % row[7] in with_table
    without = _plan_info_in_fresh_process({"PEAK_GEMM_TUNING": ""}, (256, 256, 1024))
    assert "variant=" in without
    # a shape that is not listed is the cost model's either way
    assert _plan_info_in_fresh_process({}, (777, 512, 1024)) == _plan_info_in_fresh_process({"PEAK_GEMM_TUNING": ""}, (777, 512, 1024))


def test_every_row_of_the_shipped_table_is_honoured():
    """A row the library cannot follow (a variant that does not fit the row's shape, a split it would
    clamp) is silently ignored at create: every shipped row must come back as the plan of its shape."""
    import subprocess
    import sys
    code = (
        "import sys; sys.path.insert(0, %r); import paper_2512_19018_amd as pg\n"
        "dts = {'f32': pg.PEAK_DT_F32, 'f16': pg.PEAK_DT_F16, 'bf16': pg.PEAK_DT_BF16}\n"
        "bad = []\n"
        "for l in open(%r):\n"
        "    r = l.split('#')[0].split()\n"
        "    if not r: continue\n"
        "    with pg.Plan(int(r[3]), int(r[4]), int(r[5]), dts[r[0]], int(r[1]), int(r[2])) as p:\n"
        "        i = p.info()\n"
        "    if (':%%s ' %% r[6]) not in i or ('split=%%s ' %% r[7]) not in i or ' streamk=0 ' not in i: bad.append((r, i))\n"
        "print(len(bad)); [print(b) for b in bad[:5]]\n"
        % (ROOT, os.path.join(ROOT, "paper_2512_19018_amd", "peak_gemm_tuning.txt")))
    env = dict(os.environ)
    env.pop("PEAK_GEMM_TUNING", None)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stderr
    assert r.stdout.split()[0] == "0", r.stdout


def test_plans_keep_a_stand_in_for_unaligned_operand_bases():
    # rows suit the 16-byte copies: a direct variant, with a register-staged stand-in for odd base addresses
    with pg.Plan(512, 512, 1024, pg.PEAK_DT_BF16, 0, 1) as p:
        info = p.info()
        assert re.search(r"unaligned=bf16_r\d+x\d+_nt", info), info
    # rows that do not: the selected variant takes any alignment itself
    with pg.Plan(512, 512, 1024, pg.PEAK_DT_BF16, 0, 1, lda=1027) as p:
        assert "unaligned=same" in p.info()
    # the workspace covers whichever of the two runs
    with pg.Plan(64, 64, 8192, pg.PEAK_DT_F16, 0, 1) as p:
        m = re.search(r"split=(\d+) ", p.info())
        assert p.workspace_bytes >= int(m.group(1)) * 64 * 64 * 4 if int(m.group(1)) > 1 else True


def test_compute_unit_count_comes_from_the_environment_when_given():
    # 1024 tiles: with 1024 CUs they fit one round and nothing needs splitting; the plan still is made
    a = _plan_info_in_fresh_process({"PEAK_GEMM_NUM_CU": "8", "PEAK_GEMM_TUNING": ""}, (1024, 1024, 8192))
    b = _plan_info_in_fresh_process({"PEAK_GEMM_NUM_CU": "1024", "PEAK_GEMM_TUNING": ""}, (1024, 1024, 8192))
    assert "variant=" in a and "variant=" in b
    assert "split=1 " in a                      # 16 tiles of 256x256 already fill 8 CUs twice over
    assert "split=1 " not in b                  # 1024 CUs: the K loop is cut to fill them


def test_calibration_calls_check_their_arguments():
    # argument checks come before any device call
    assert pg.peak_calib_mfma(7, True, 10, 0x1000)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_mfma(pg.PEAK_DT_BF16, True, 0, 0x1000)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_mfma(pg.PEAK_DT_BF16, True, 10, 0)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_mfma(pg.PEAK_DT_BF16, True, 10, 0x1004)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_read(0, 1 << 20, 0x1000) == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_read(0x1008, 1 << 20, 0x1000) == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_read(0x1000, 8, 0x1000) == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_lds_load(0, 1 << 30, 10, 0x1000)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_lds_load(0x1000, 1 << 30, 0, 0x1000)[0] == pg.PEAK_ERR_INVALID_ARG
    assert pg.peak_calib_lds_load(0x1000, 1 << 30, 10, 0x1004)[0] == pg.PEAK_ERR_INVALID_ARG


def test_hybrid_stream_k_plans():
    """576 tiles of 256x256 on 256 compute units: two full rounds and 64 tiles over.  The cut
    round: 64 tiles x 4 K slices, dense fp32 partial tiles in the workspace."""
    env = {"PEAK_GEMM_NUM_CU": "256", "PEAK_GEMM_TUNING": ""}
    code = ("import sys; sys.path.insert(0, %r); import paper_2512_19018_amd as pg\n"
            "for sk in (True, False, None):\n"
            "    with pg.Plan(8192, 4608, 8192, pg.PEAK_DT_BF16, 0, 1, flags=pg.force_flags(streamk=sk)) as p: print(p.info(), p.workspace_bytes)\n"
            "with pg.Plan(8192, 8192, 8192, pg.PEAK_DT_BF16, 0, 1, flags=pg.force_flags(streamk=True)) as p: print(p.info(), p.workspace_bytes)\n"
            "with pg.Plan(8192, 4608, 8192, pg.PEAK_DT_BF16, 0, 1, flags=pg.force_flags(split=2, streamk=True)) as p: print(p.info(), p.workspace_bytes)\n"
            "with pg.Plan(8192, 4608, 8192, pg.PEAK_DT_F32, 0, 1, flags=pg.force_flags(streamk=True)) as p: print(p.info(), p.workspace_bytes)\n" % ROOT)
    import subprocess
    import sys
    e = dict(os.environ)
    e.update(env)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120, env=e)
    assert r.returncode == 0, r.stderr
    on, off, auto, exact, forced_split, f32 = r.stdout.strip().split("\n")
    assert "bf16_m256x256w4a3_nt" in on and "streamk=64" in on and "split=4 " in on and "ktiles/slice=32" in on
    assert "grid=%d " % (512 + 64 * 4) in on and on.endswith(" %d" % (4 * 64 * 256 * 256 * 4))
    assert "streamk=0" in off and "split=1 " in off and off.endswith(" 0")
    assert "streamk=64" in auto                              # a quarter round for a whole one: the cost model takes it
    assert "streamk=0" in exact and "split=1 " in exact      # 1024 tiles: four whole rounds, nothing to cut
    assert "streamk=0" in forced_split and "split=2 " in forced_split
    assert "streamk=0" in f32                                # the fp32 kernels do not have it


def test_streaming_plans_cover_m_up_to_64_fp32_and_b_stored_k_by_n():
    """Skinny products (M <= 64) whose big operand can be streamed once go to a streaming
    kernel: fewest 16-row blocks that hold M, fp32 as well as 16-bit storage, B along K or
    stored K x N; other shapes and layouts stay with the tiled kernels."""
    def info(M, N, K, dt, tA, tB):
        with pg.Plan(M, N, K, dt, tA, tB) as p:
            return p.info()
    bf, f16, f32 = pg.PEAK_DT_BF16, pg.PEAK_DT_F16, pg.PEAK_DT_F32
    assert "bf16_skinny128k256s2_nt" in info(16, 28672, 8192, bf, 0, 1)
    assert "split=1 " in info(16, 28672, 8192, bf, 0, 1)              # 224 workgroups on 256 CUs: no K split
    assert "skinny_m32n128" in info(17, 28672, 8192, bf, 0, 1)
    assert "skinny_m32n64" in info(32, 4096, 4096, f16, 0, 1)
    assert "skinny_m64n128" in info(33, 8192, 28672, bf, 0, 1)        # tall M x K operand: 128 rows per workgroup even when split
    assert "skinny_m64n128" in info(64, 28672, 8192, f16, 0, 1)
    assert "skinny" not in info(65, 28672, 8192, bf, 0, 1)
    assert "f32_skinny_m16" in info(16, 16384, 16384, f32, 0, 1)
    assert "f32_skinny_m64n64k64s3w8p_nt" in info(64, 16384, 8192, f32, 0, 1)    # MFMA bound: two waves per 16 rows, pipelined loop
    assert "f32_skinny_m32n64k64s3w8p_nt" in info(24, 16384, 8192, f32, 0, 1)
    # B stored K x N
    assert "bf16_skinny_m16n256k64s4_nn" in info(16, 28672, 8192, bf, 0, 0)
    assert "f16_skinny_m64n256k64s4_nn" in info(48, 28672, 8192, f16, 0, 0)
    assert "f32_skinny_m32n128k32s6_nn" in info(20, 16384, 8192, f32, 0, 0)
    assert "skinny" not in info(16, 28668, 8192, bf, 0, 0)            # N not a whole number of 16-byte chunks
    assert "skinny" not in info(16, 28672, 8200, bf, 0, 0)            # K not a whole number of stages
    # A stored K x M: the same kernels on a copy of A written out along K, which the workspace holds
    # behind the Split-K partials (256-byte boundary); not for a streamed operand of a few MB
    tt, tn = info(16, 28672, 8192, bf, 1, 1), info(40, 28672, 8192, f32, 1, 0)
    assert "bf16_skinny" in tt and tt.endswith("acopy=1") and "f32_skinny_m64n128k32s6_nn" in tn and tn.endswith("acopy=1")
    assert info(16, 28672, 8192, bf, 0, 1).endswith("acopy=0")
    with pg.Plan(16, 28672, 8192, bf, 1, 1, flags=pg.force_flags(split=2)) as p:
        assert p.info().endswith("acopy=1") and p.workspace_bytes >= 2 * 16 * 28672 * 4 + 16 * 8192 * 2
    assert "skinny" not in info(16, 1024, 1024, bf, 1, 1) and "skinny" not in info(65, 28672, 8192, bf, 1, 1)
    assert "skinny" not in info(16, 28672, 8200, bf, 1, 1)


def test_tile_order_and_k_rotation_of_the_plans():
    """Bands of four tile rows where the problem has 16 or more tile columns, eight otherwise; the
    16x16x32 kernels start their workgroups one K tile apart when there is a single row of tiles
    (every workgroup then streams rows of B that no other reads), the streaming NT kernel five apart."""
    def info(M, N, K, dt, tA, tB):
        with pg.Plan(M, N, K, dt, tA, tB) as p:
            return p.info()
    bf, f16 = pg.PEAK_DT_BF16, pg.PEAK_DT_F16
    c3 = info(8192, 8192, 8192, bf, 0, 1)
    assert "group_m=4 " in c3 and " rot=0,0 " in c3
    c4 = info(5000, 3000, 12288, f16, 0, 0)
    assert "group_m=8 " in c4 and " rot=0,0 " in c4
    single = info(128, 28672, 8192, bf, 0, 1)
    assert "_m128x128" in single and "(tiles 1x224)" in single and " rot=0,1 " in single
    assert " rot=0,5 " in info(16, 16384, 16384, bf, 0, 1)
    assert " rot=0,0 " in info(16, 28672, 8192, bf, 0, 0)        # B stored K x N: contiguous pieces of a k-row
