"""Offline exhaustive sweep over the library's kernel variants and K splits.

The paper's "performance evaluators" (Section 3.3) enumerate the valid values
of a kernel's tuning parameters, time each setting and keep the best; settings
the kernel context rejects are skipped (Section 3.1, the invalid-configuration
sentinel).  Here the tuning parameters are the kernel variant (tile, waves,
staging scheme, ring depth) and the K split; `peak_gemm_create` with the force
bits set is the validity check (PEAK_ERR_UNSUPPORTED = skip), and the result
is a selector table that `peak_gemm_load_tuning` / PEAK_GEMM_TUNING feed back
into the library.

    python -m paper_2512_19018_amd.tune --shape bf16:0:1:8192:8192:8192 --out table.txt
    python -m paper_2512_19018_amd.tune --workloads C3 C4 --out table.txt

Needs a GPU; torch is used for device memory, random fill and events only.
"""
from __future__ import annotations

import argparse
import sys
import time

from . import binding as pg

DT_NAMES = {"f32": pg.PEAK_DT_F32, "f16": pg.PEAK_DT_F16, "bf16": pg.PEAK_DT_BF16}
DT_OF = {v: k for k, v in DT_NAMES.items()}
SPLITS = (1, 2, 3, 4, 6, 8, 12, 16, 32)


def candidates(dtype, transA, transB, M, N, K, lda=None, ldb=None, ldc=None, splits=SPLITS):
    """(variant id, name, split, plan info) of every setting the library accepts
    for the problem.  A split the plan would clamp to a smaller one is listed once."""
    out, seen = [], set()
    for vid in range(pg.peak_gemm_variant_count()):
        name = pg.peak_gemm_variant_name(vid)
        for split in splits:
            try:
                plan = pg.Plan(M, N, K, dtype, transA, transB, lda, ldb, ldc, pg.force_flags(vid, split))
            except pg.PeakError as e:
                if e.status == pg.PEAK_ERR_UNSUPPORTED:
                    break                    # the variant does not fit this problem at all
                raise
            info = plan.info()
            eff = int(info.split("split=")[1].split()[0])
            plan.close()
            if (vid, eff) in seen:
                continue
            seen.add((vid, eff))
            out.append((vid, name, eff, info))
    return out


def time_setting(torch, plan, alpha, beta, dA, dB, dC, reps, warmup):
    ws = torch.empty(max(plan.workspace_bytes, 4), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    args = (alpha, dA.data_ptr(), dB.data_ptr(), beta, dC.data_ptr(), ws.data_ptr(), plan.workspace_bytes,
            stream.cuda_stream)
    for _ in range(warmup):
        plan.run(*args)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        plan.run(*args)
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps          # microseconds per launch


def sweep(dtype, transA, transB, M, N, K, alpha=1.0, beta=0.0, reps=20, warmup=3, splits=SPLITS, log=None):
    """Time every accepted setting; returns a list of (us, name, split) sorted by time."""
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("tune.sweep needs a GPU")
    tdt = {pg.PEAK_DT_F32: torch.float32, pg.PEAK_DT_F16: torch.float16, pg.PEAK_DT_BF16: torch.bfloat16}[dtype]
    scale = 1.0 / max(K, 1) ** 0.5
    dA = (torch.randn((K, M) if transA else (M, K), device="cuda") * scale).to(tdt)
    dB = (torch.randn((N, K) if transB else (K, N), device="cuda") * scale).to(tdt)
    dC = torch.zeros((M, N), device="cuda", dtype=tdt)
    results = []
    for vid, name, split, info in candidates(dtype, transA, transB, M, N, K, splits=splits):
        with pg.Plan(M, N, K, dtype, transA, transB, flags=pg.force_flags(vid, split)) as plan:
            us = time_setting(torch, plan, alpha, beta, dA, dB, dC, reps, warmup)
        results.append((us, name, split))
        if log:
            log("  %-32s split=%-3d %10.1f us" % (name, split, us))
    results.sort()
    return results


def own_choice(dtype, transA, transB, M, N, K):
    """(variant name, split) of the plan the library makes by itself for the problem (cost model, or
    whatever selector table is loaded: run the sweep with PEAK_GEMM_TUNING="" to have the model's)."""
    with pg.Plan(M, N, K, dtype, transA, transB) as plan:
        info = plan.info()
    return info.split("variant=")[1].split()[0].split(":", 1)[1], int(info.split("split=")[1].split()[0])


def time_own(dtype, transA, transB, M, N, K, alpha=1.0, beta=0.0, reps=20, warmup=3):
    """(us, plan info) of the plan the library makes by itself, timed like the sweep's settings.  A plan with
    hybrid stream-K (only part of the tiles cut along K) has no forced counterpart in the sweep, and the
    table's (variant, split) rows cannot ask for it."""
    import torch
    tdt = {pg.PEAK_DT_F32: torch.float32, pg.PEAK_DT_F16: torch.float16, pg.PEAK_DT_BF16: torch.bfloat16}[dtype]
    scale = 1.0 / max(K, 1) ** 0.5
    dA = (torch.randn((K, M) if transA else (M, K), device="cuda") * scale).to(tdt)
    dB = (torch.randn((N, K) if transB else (K, N), device="cuda") * scale).to(tdt)
    dC = torch.zeros((M, N), device="cuda", dtype=tdt)
    with pg.Plan(M, N, K, dtype, transA, transB) as plan:
        return time_setting(torch, plan, alpha, beta, dA, dB, dC, reps, warmup), plan.info()


def is_streamk(info):
    """True when the plan description says that part of the tiles are cut into K slices."""
    return "streamk=" in info and int(info.split("streamk=")[1].split()[0]) > 0


def pick(results, own, margin):
    """The row to write for a problem: the library's own choice when it is within `margin` of the
    fastest setting (differences that small are run-to-run noise, and a table that follows them
    changes with every sweep), else the fastest."""
    best = results[0]
    for us, name, split in results:
        if (name, split) == own and us <= best[0] * (1.0 + margin):
            return us, name, split
    return best


def table_line(dtype, transA, transB, M, N, K, name, split, us):
    return "%s %d %d %d %d %d %s %d   # %.1f us" % (DT_OF[dtype], transA, transB, M, N, K, name, split, us)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--shape", action="append", default=[], metavar="DT:TA:TB:M:N:K",
                    help="problem to tune, e.g. bf16:0:1:8192:8192:8192 (repeatable)")
    ap.add_argument("--workloads", nargs="*", default=[], help="named workloads of peak_inputs (C1..C5, P2k_f32, ...)")
    ap.add_argument("--out", default=None, help="selector table to write (default: stdout)")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--margin", type=float, default=0.015,
                    help="keep the library's own choice when it is within this fraction of the fastest setting")
    args = ap.parse_args(argv)

    problems = []
    for s in args.shape:
        dt, ta, tb, M, N, K = s.split(":")
        problems.append((DT_NAMES[dt], int(ta), int(tb), int(M), int(N), int(K), 1.0, 0.0))
    if args.workloads:
        import peak_inputs as pi
        for name in args.workloads:
            w = pi.WORKLOADS[name]
            problems.append((w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, w.beta))
    if not problems:
        ap.error("nothing to tune: give --shape or --workloads")

    def log(msg):
        print(msg, file=sys.stderr, flush=True)

    lines = ["# selector table written by paper_2512_19018_amd.tune on %s" % time.strftime("%Y-%m-%d"),
             "# dtype transA transB M N K variant split"]
    for dtype, ta, tb, M, N, K, alpha, beta in problems:
        log("%s transA=%d transB=%d %dx%dx%d" % (DT_OF[dtype], ta, tb, M, N, K))
        res = sweep(dtype, ta, tb, M, N, K, alpha, beta, args.reps, args.warmup, log=log)
        own_us, own_info = time_own(dtype, ta, tb, M, N, K, alpha, beta, args.reps, args.warmup)
        if is_streamk(own_info) and own_us <= res[0][0] * (1.0 + args.margin):
            # a row would switch the stream-K plan off: leave the problem to the library's own choice
            log("  own stream-K plan %.1f us, fastest forced setting %.1f us: no row" % (own_us, res[0][0]))
            lines.append("# %s %d %d %d %d %d: the library's own stream-K plan (%.1f us) is left in place"
                         % (DT_OF[dtype], ta, tb, M, N, K, own_us))
            continue
        us, name, split = pick(res, own_choice(dtype, ta, tb, M, N, K), args.margin)
        log("  best: %s split=%d %.1f us (of %d settings; fastest %s split=%d %.1f us)" % ((name, split, us, len(res)) + (res[0][1], res[0][2], res[0][0])))
        lines.append(table_line(dtype, ta, tb, M, N, K, name, split, us))
    text = "\n".join(lines) + "\n"
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)


if __name__ == "__main__":
    main()
