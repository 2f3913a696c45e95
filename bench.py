#!/usr/bin/env python3
"""Bench of the GEMM hot path on one MI355X.

A "step" is one pass of the whole hot path (plan already made; tile schedule,
staging, MFMA loop, split-K reduction where used, epilogue) over one seeded
synthetic problem already resident in HBM.  The headline workload is the bf16
8192^3 NT product (C3); the other workloads are timed the same way and listed
under "workloads" in the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--only] [--no-cpu] [--no-torch]

Order of a run: the headline workload's inputs are made and uploaded; the
matrix cores' sustained rate is measured with an MFMA-only loop on random
operands (include/peak_calib.h); launches of the workload itself for --settle-ms
(the chip's power management takes some 50 launches to settle after a change of
load, and the calibration loop is a different load; the count is in the line as
"settle_launches"); then W warmup steps, K timed steps between one pair of HIP events, K more steps with an event pair each (median, min, mean);
torch.matmul on the same buffers as context; the CPU oracle on a bounded sample
of rows; then the other workloads the same way with shorter CPU samples.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0

# Bytes per launch that cross the L2 <-> memory boundary, from rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE (profiles/*_summary.md), each scaled by what the same
# counter reads for a plain 1 GiB device copy (FETCH_SIZE reads half the bytes:
# factor 2.0; WRITE_SIZE factor 1.0).  Summed over the kernels of one launch.
# A figure belongs to the kernel variant it was measured on: it is reported only
# when the plan of this run selects that very variant and split, else null.
MEASURED_TRAFFIC = {
    "C3": ("bf16_m256x256w4a3_nt", 1, 1.746e9),
    "C3b": ("bf16_m256x256w4a3_nt", 1, 2.352e8),
    "C5": ("bf16_skinny16s3_nt", 1, 5.569e8),
    "C2": ("f32_t256x256w4a3_nn", 1, 5.380e8),
    "C4": ("f16_m256x256w4a3_nn", 1, 7.340e8),
    "S16_bf16_kn": ("bf16_skinny_m16n256k64s4_nn", 2, 4.803e8),
    "S64_f16": ("f16_skinny_m64n128k128s3_nt", 1, 5.401e8),
    "S16_f32": ("f32_skinny_m16n64k128s3_nt", 1, 1.2091e9),
    "P2k_f16": ("f16_m128x128k128w4a3_nn", 1, 5.90e7),
    "D128_bf16": ("bf16_m128x128k128w4a3_nt", 1, 5.088e8),
    "S64_f32": ("f32_skinny_m64n64k64s3w8p_nt", 1, 8.088e8),
}


def measured_traffic(name, plan_info):
    t = MEASURED_TRAFFIC.get(name)
    if not t:
        return None
    variant, split, nbytes = t
    return nbytes if (":%s " % variant) in plan_info and ("split=%d " % split) in plan_info else None


def smi_snapshot():
    """Clocks and power as rocm-smi reports them (a child process; context only)."""
    import shutil
    import subprocess
    try:
        # rocm-smi is a script: run it with this interpreter (no re-exec through env), and without a
        # profiler's preloaded tool library, which would initialise the GPU in the child as well
        tool = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
        env = {k: v for k, v in os.environ.items()
               if k not in ("LD_PRELOAD", "HSA_TOOLS_LIB", "ROCP_TOOL_LIBRARIES") and not k.startswith("ROCPROF")}
        r = subprocess.run([sys.executable, tool, "--showclocks", "--showpower", "--json"], capture_output=True, text=True,
                           timeout=30, env=env)
        d = json.loads(r.stdout)
        card = d[sorted(d)[0]]
        keep = {}
        for k, v in card.items():
            kl = k.lower()
            if "sclk" in kl or "mclk" in kl or "power" in kl:
                keep[k] = v
        return keep or None
    except Exception as ex:
        return {"error": repr(ex)[:120]}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clocks of an idle chip take some 50 launches of the headline workload to settle (measured:
    # 1367 TFLOP/s after 10 warmup steps, 1397 after 50, 1400-1409 after 200); the default warmup
    # is long enough that the timed steps see the sustained state
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="before the W warmup steps: launches of the workload for this long (at most 2000), so that a "
                         "short warmup does not time the power management's reaction to the change of load")
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--only", action="store_true", help="time only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-torch", action="store_true", help="skip the torch.matmul context rows")
    ap.add_argument("--variant", default=None, help="force a kernel variant, by id or name (sweeps)")
    ap.add_argument("--split", type=int, default=None, help="force a K split (sweeps)")
    ap.add_argument("--fused", choices=["gelu", "relu"], default=None,
                    help="time peak_gemm_run_fused (bias per column + tanh-form GELU or ReLU) instead of peak_gemm_run")
    ap.add_argument("--fast-inputs", action="store_true",
                    help="sweeps only: random device-generated inputs instead of the seeded host generator")
    ap.add_argument("--constant-inputs", action="store_true",
                    help="diagnostic only: every element 1.0 (the matrix pipe then draws far less power; shows how "
                         "much of the time is the chip's power limit)")
    ap.add_argument("--no-calibration", action="store_true",
                    help="skip the MFMA-only / read-only calibration legs (profiling runs that want the GEMM kernels only)")
    ap.add_argument("--alternate-library", type=float, default=None, metavar="SECONDS",
                    help="instead of the bench: blocks of SECONDS of this library, of torch.matmul and of the MFMA-only "
                         "loop in turn on the workload's shape, with rocm-smi clock and power sampled during each "
                         "(box-independent comparison, and the record of the power limit)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy instead (to scale FETCH_SIZE / WRITE_SIZE under rocprofv3)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the GEMM kernel on one GPU's share); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import peak_inputs as pi
    import paper_2512_19018_amd as pg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    pg.load_library()          # no fallback: raises if the HIP library is not built
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        n = 1 << 30
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": args.steps}))
        return

    if args.alternate_library:
        import threading
        import time as _time
        w = pi.WORKLOADS[args.workload]
        tdt = {pi.F32: torch.float32, pi.F16: torch.float16, pi.BF16: torch.bfloat16}[w.dtype]
        A = (torch.randn((w.K, w.M) if w.transA else (w.M, w.K), device="cuda") * w.scale).to(tdt)
        B = (torch.randn((w.N, w.K) if w.transB else (w.K, w.N), device="cuda") * w.scale).to(tdt)
        C = torch.zeros((w.M, w.N), device="cuda", dtype=tdt)
        opA, opB, out = (A.t() if w.transA else A), (B.t() if w.transB else B), torch.empty_like(C)
        calib = torch.zeros(8, dtype=torch.int64, device="cuda")
        samples, stop = [], [False]

        def sampler():
            while not stop[0]:
                samples.append((_time.time(), smi_snapshot()))

        th = threading.Thread(target=sampler, daemon=True)
        th.start()
        blocks = []

        def block(label, fn, seconds, flops):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0, rates = _time.time(), []
            while _time.time() - t0 < seconds:
                e0.record(stream)
                for _ in range(20):
                    fn()
                e1.record(stream)
                e1.synchronize()
                rates.append(flops * 20 / (e0.elapsed_time(e1) * 1e-3) * 1e-12)
            t1 = _time.time()
            smi = [x[1] for x in samples if t0 + 0.5 < x[0] < t1]
            blocks.append({"what": label, "tflops_median": float(np.median(rates)), "tflops_last": rates[-1], "batches": len(rates),
                           "rocm_smi_last": smi[-1] if smi else None})
            log("[alternate] %-14s %8.1f TFLOP/s  %s" % (label, blocks[-1]["tflops_median"], blocks[-1]["rocm_smi_last"]))

        with pg.Plan(w.M, w.N, w.K, w.dtype, w.transA, w.transB) as plan:
            ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
            _, mfma_flops = pg.peak_calib_mfma(w.dtype, True, 4096, calib.data_ptr(), stream.cuda_stream)
            for rnd in range(2):
                block("mfma_only", lambda: pg.peak_calib_mfma(w.dtype, True, 4096, calib.data_ptr(), stream.cuda_stream), 1.0, mfma_flops)
                block("this_library", lambda: plan.run(w.alpha, A.data_ptr(), B.data_ptr(), 0.0, C.data_ptr(), ws.data_ptr(),
                                                       plan.workspace_bytes, stream.cuda_stream), args.alternate_library, w.flops)
                block("torch_matmul", lambda: torch.matmul(opA, opB, out=out), args.alternate_library, w.flops)
            info = plan.info()
        stop[0] = True
        print(json.dumps({"alternate_library": args.workload, "plan": info, "blocks": blocks}))
        return

    def dev(x):
        return torch.from_numpy(x.view(np.int16).copy() if x.dtype == np.uint16 else np.ascontiguousarray(x)).cuda()

    calib_out = torch.zeros(8, dtype=torch.int64, device="cuda")
    sustained = {}          # dtype name -> {"tflops", "clock_ghz"}: MFMA-only loop, random operands

    def mfma_sustained(dtype):
        """What the matrix cores sustain on this machine right now: the MFMA-only loop of
        include/peak_calib.h on random operands, about a quarter of a second of it."""
        name = pi.DTYPE_NAMES[dtype]
        iters = 4096 if dtype != pi.F32 else 2048
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = None
        for rep in range(4):
            launches = 40
            e0.record(stream)
            for _ in range(launches):
                st, flops = pg.peak_calib_mfma(dtype, True, iters, calib_out.data_ptr(), stream.cuda_stream)
                if st != pg.PEAK_OK:
                    raise SystemExit("bench.py: peak_calib_mfma: " + pg.peak_status_string(st))
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / launches
            c = calib_out.cpu().numpy()
            best = {"tflops": flops / (ms * 1e-3) * 1e-12, "clock_ghz": 0.1 * float(c[0]) / max(float(c[1]), 1.0)}
        sustained[name] = best          # the last repetition: the settled state
        return best

    read_stream = {}

    def hbm_read_sustained():
        """Read bandwidth a kernel gets that only reads: 2 GiB, far beyond the last-level cache."""
        n = 1 << 31
        src = torch.empty(n, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for rep in range(2):
            launches = 10
            e0.record(stream)
            for _ in range(launches):
                st = pg.peak_calib_read(src.data_ptr(), n, calib_out.data_ptr(), stream.cuda_stream)
                if st != pg.PEAK_OK:
                    raise SystemExit("bench.py: peak_calib_read: " + pg.peak_status_string(st))
            e1.record(stream)
            e1.synchronize()
            read_stream["gbs"] = n / (e0.elapsed_time(e1) / launches * 1e-3) * 1e-9
        del src
        torch.cuda.empty_cache()
        return read_stream["gbs"]

    lds_path = {}

    def lds_load_rate():
        """Bytes per cycle one compute unit's path from the L2 into LDS delivers (direct-to-LDS loads and
        nothing else, include/peak_calib.h): the second ceiling of a tiled kernel, next to the MFMA rate."""
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        src = torch.empty(cus * 64 * 1024, dtype=torch.uint8, device="cuda")
        src.random_(0, 255)
        out = torch.zeros(2 * cus, dtype=torch.int64, device="cuda")
        for rep in range(2):                                 # the second launch finds its pieces in the L2
            st, nbytes, wgs = pg.peak_calib_lds_load(src.data_ptr(), src.numel(), 2000, out.data_ptr(), stream.cuda_stream)
            if st != pg.PEAK_OK:
                raise SystemExit("bench.py: peak_calib_lds_load: " + pg.peak_status_string(st))
            stream.synchronize()
        c = out.cpu().numpy().reshape(-1, 2)
        lds_path["bytes_per_cycle_per_cu"] = float(nbytes / c[:wgs, 0].mean())
        return lds_path["bytes_per_cycle_per_cu"]

    def cpu_leg(w, host, seconds, threads=None, label=None):
        """The oracle as it stands on a bounded sample of rows of C (all columns, full K)."""
        from oracle import gemm_oracle
        A, B, C = host
        threads = threads or gemm_oracle.default_threads()
        cin = C if w.beta != 0 else None
        t0 = time.perf_counter()
        gemm_oracle.gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, w.beta, cin,
                         rows=list(range(min(threads, w.M))), threads=threads)
        t_probe = time.perf_counter() - t0
        nrows = int(max(threads, min(w.M, threads * max(1.0, seconds / max(t_probe, 1e-4)))))
        nrows = min(w.M, (nrows // threads) * threads if nrows >= threads else nrows)
        rows = [int(r) for r in np.linspace(0, w.M - 1, nrows).astype(np.int64)]
        t0 = time.perf_counter()
        gemm_oracle.gemm(w.dtype, w.transA, w.transB, w.M, w.N, w.K, w.alpha, A, B, w.beta, cin, rows=rows, threads=threads)
        t_cpu = time.perf_counter() - t0
        return {"value": 2.0 * len(rows) * w.N * w.K / t_cpu * 1e-12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                "sample": "%d of %d rows of C (all N columns, full K) of %s in %.2f s on %d thread%s; rate scaled to the "
                          "whole product" % (len(rows), w.M, label or w.name, t_cpu, threads, "" if threads == 1 else "s")}

    def settle(launch):
        """Launches in groups of ten until --settle-ms have passed (at most 2000); returns the count."""
        n = 0
        t0 = time.perf_counter()
        while args.settle_ms > 0 and n < 2000 and (time.perf_counter() - t0) * 1e3 < args.settle_ms:
            for _ in range(10):
                launch(n)
                n += 1
            torch.cuda.synchronize()
        return n

    def time_workload(name, steps, warmup, variant=None, split=None, with_torch=True, cpu_seconds=0.0):
        w = pi.WORKLOADS[name]
        t0 = time.time()
        if args.fast_inputs or args.constant_inputs:
            tdt0 = {pi.F32: torch.float32, pi.F16: torch.float16, pi.BF16: torch.bfloat16}[w.dtype]

            def rnd(r, c):
                t = (torch.ones(r, c, device="cuda") if args.constant_inputs
                     else torch.randn(r, c, device="cuda") * w.scale).to(tdt0)
                t = t.view(torch.int16) if w.dtype != pi.F32 else t
                a = t.cpu().numpy()
                return a.view(np.uint16) if w.dtype != pi.F32 else a
            A = rnd(*( (w.K, w.M) if w.transA else (w.M, w.K) ))
            B = rnd(*( (w.N, w.K) if w.transB else (w.K, w.N) ))
            C = rnd(w.M, w.N)
        else:
            A, B, C = w.make(with_cin=True)
        log("[bench] %s: inputs generated in %.1f s" % (name, time.time() - t0))
        # rotate buffer sets for problems that would otherwise sit in the 256 MB last-level cache
        nset = 1
        footprint = A.nbytes + B.nbytes + C.nbytes
        if footprint < 600e6:
            nset = int(min(8, max(2, 600e6 // footprint + 1)))
        dA = [dev(A) for _ in range(nset)]
        dB = [dev(B) for _ in range(nset)]
        dC = [dev(C) for _ in range(nset)]
        lda, ldb, ldc = w.ld()
        if variant is not None and not str(variant).isdigit():
            names = [pg.peak_gemm_variant_name(i) for i in range(pg.peak_gemm_variant_count())]
            if variant not in names:
                raise SystemExit("bench.py: no kernel variant named %r" % (variant,))
            variant = names.index(variant)
        flags = pg.force_flags(None if variant is None else int(variant), split)
        dname = pi.DTYPE_NAMES[w.dtype]
        res = {"workload": name, "note": w.note, "dtype": dname, "M": w.M, "N": w.N, "K": w.K,
               "transA": w.transA, "transB": w.transB, "alpha": w.alpha, "beta": w.beta, "buffer_sets": nset}
        hbm_bound = (w.flops / w.min_bytes) < (PEAK_TFLOPS[dname] * 1e12 / (PEAK_HBM_GBS * 1e9))
        if not args.no_calibration:
            # the ceiling first, in the state the timed steps will find
            if hbm_bound:
                if "gbs" not in read_stream:
                    hbm_read_sustained()
            else:
                if not lds_path:
                    lds_load_rate()
                mfma_sustained(w.dtype)                      # last: it leaves the chip in the state of a matrix load
        with pg.Plan(w.M, w.N, w.K, w.dtype, w.transA, w.transB, lda, ldb, ldc, flags) as plan:
            res["plan"] = plan.info()
            ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")

            if args.fused:
                res["fused"] = "bias per column + " + args.fused
                act = pg.PEAK_ACT_GELU_TANH if args.fused == "gelu" else pg.PEAK_ACT_RELU
                dbias = (torch.rand(w.N, device="cuda", dtype=torch.float32) - 0.5)

            def step(i):
                s = i % nset
                if args.fused:
                    plan.run_fused(w.alpha, dA[s].data_ptr(), dB[s].data_ptr(), w.beta, dC[s].data_ptr(),
                                   pg.PEAK_BIAS_PER_COLUMN, dbias.data_ptr(), act,
                                   ws.data_ptr(), plan.workspace_bytes, stream.cuda_stream)
                else:
                    plan.run(w.alpha, dA[s].data_ptr(), dB[s].data_ptr(), w.beta, dC[s].data_ptr(),
                             ws.data_ptr(), plan.workspace_bytes, stream.cuda_stream)

            res["settle_launches"] = settle(step)
            for i in range(warmup):
                step(i)
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record(stream)
            for i in range(steps):
                step(i)
            e1.record(stream)
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3 / steps
            ev_ms = e0.elapsed_time(e1) / steps
            # the same number of launches again, an event pair around each
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for i, (a0, a1) in enumerate(pairs):
                a0.record(stream)
                step(i)
                a1.record(stream)
            torch.cuda.synchronize()
            each = np.array([a0.elapsed_time(a1) for a0, a1 in pairs])
        res["ms_per_step"] = wall_ms
        res["event_ms_per_step"] = ev_ms
        res["per_launch_ms"] = {"median": float(np.median(each)), "min": float(each.min()), "mean": float(each.mean()),
                                "launches": int(each.size)}
        res["tflops"] = w.flops / (wall_ms * 1e-3) * 1e-12
        res["tflops_events"] = w.flops / (ev_ms * 1e-3) * 1e-12
        res["gbs_events"] = w.min_bytes / (ev_ms * 1e-3) * 1e-9
        traffic = measured_traffic(name, res["plan"])
        if hbm_bound:
            res["roofline"] = {"bound": "hbm", "achieved": res["gbs_events"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": res["gbs_events"] / PEAK_HBM_GBS, "traffic": traffic}
            if "gbs" in read_stream:
                res["roofline"]["read_only_stream_gbs"] = read_stream["gbs"]
                res["roofline"]["frac_of_read_only_stream"] = res["gbs_events"] / read_stream["gbs"]
        else:
            pk = PEAK_TFLOPS[dname]
            res["roofline"] = {"bound": "mfma", "achieved": res["tflops_events"], "peak": pk, "unit": "TFLOP/s",
                               "frac": res["tflops_events"] / pk, "traffic": traffic}
            if dname in sustained:
                # the data-sheet peak assumes 2.4 GHz; under an MFMA-only load with random operands the
                # chip holds clock_ghz, and peak * clock_ghz / 2.4 is what it can issue in that state
                sus = sustained[dname]
                res["roofline"]["mfma_only_sustained"] = sus["tflops"]
                res["roofline"]["mfma_only_clock_ghz"] = sus["clock_ghz"]
                res["roofline"]["peak_at_measured_clock"] = pk * sus["clock_ghz"] / 2.4
                res["roofline"]["frac_measured_clock"] = res["tflops_events"] / (pk * sus["clock_ghz"] / 2.4)
            if lds_path:
                # what the tile of the plan asks of the L2 -> LDS path at the full MFMA rate, against what the
                # path delivers: bytes of A and B per K tile over the cycles its MFMAs take on four SIMDs
                import re
                m = re.search(r"tile=(\d+)x(\d+)x(\d+)", res["plan"])
                if m:
                    bm, bn, bk = (int(x) for x in m.groups())
                    es = pi.DTYPE_SIZE[w.dtype]
                    flops_per_cycle_cu = pk * 1e12 / (2.4e9 * 256)
                    need = (bm + bn) * bk * es / (2.0 * bm * bn * bk / flops_per_cycle_cu)
                    res["roofline"]["l2_to_lds_bytes_per_cycle_per_cu"] = lds_path["bytes_per_cycle_per_cu"]
                    res["roofline"]["tile_needs_bytes_per_cycle_per_cu"] = need
        if with_torch:
            try:
                tdt = {pi.F32: torch.float32, pi.F16: torch.float16, pi.BF16: torch.bfloat16}[w.dtype]
                tA = dA[0].view(tdt) if w.dtype != pi.F32 else dA[0]
                tB = dB[0].view(tdt) if w.dtype != pi.F32 else dB[0]
                tC = dC[0].view(tdt) if w.dtype != pi.F32 else dC[0]
                opA = tA.t() if w.transA else tA
                opB = tB.t() if w.transB else tB
                out = torch.empty_like(tC)

                def tstep():
                    if w.beta != 0:
                        torch.addmm(tC, opA, opB, beta=w.beta, alpha=w.alpha, out=out)
                    else:
                        torch.matmul(opA, opB, out=out)
                settle(lambda i: tstep())
                for _ in range(max(3, warmup // 2)):
                    tstep()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    tstep()
                torch.cuda.synchronize()
                tms = (time.perf_counter() - t0) * 1e3 / steps
                res["torch_ms"] = tms
                res["torch_tflops"] = w.flops / (tms * 1e-3) * 1e-12
                res["pct_of_library"] = 100.0 * res["tflops"] / res["torch_tflops"]
            except Exception as ex:      # context only
                res["torch_error"] = repr(ex)[:200]
        del dA, dB, dC
        torch.cuda.empty_cache()
        if cpu_seconds > 0:
            res["cpu_baseline"] = cpu_leg(w, (A, B, C), cpu_seconds)
            if name in ("C1", "C5"):
                res["cpu_baseline_1_thread"] = cpu_leg(w, (A, B, C), min(cpu_seconds, 3.0), threads=1)
        return res, (A, B, C)

    smi_before = smi_snapshot()
    head, host = time_workload(args.workload, args.steps, args.warmup, args.variant, args.split,
                               with_torch=not args.no_torch)
    w = pi.WORKLOADS[args.workload]

    out = {
        "metric": "GEMM TFLOP/s and % of MFMA peak (bf16 8192^3; fp32 4096^3) on 1 MI355X",
        "value": head["tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic (seeded splitmix64 counters; see peak_inputs)",
        "config": {"workload": "%s: %s, M=%d N=%d K=%d transA=%d transB=%d alpha=%g beta=%g"
                               % (w.name, w.note, w.M, w.N, w.K, w.transA, w.transB, w.alpha, w.beta),
                   "plan": head["plan"]},
        "roofline": head["roofline"],
        "pct_of_peak": 100.0 * head["roofline"]["frac"],
        "per_launch_ms": head["per_launch_ms"],
        "settle_launches": head["settle_launches"],
        "torch_matmul_tflops": head.get("torch_tflops"),
        "pct_of_library": head.get("pct_of_library"),
    }

    # CPU baseline: the oracle as it stands, on a bounded sample of rows of the same workload
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_leg(w, host, 15.0)
    del host

    if not args.only:
        others = []
        for name in ["C1", "C2", "C3b", "C4", "C5", "P2k_f32", "P4k_f32", "P2k_f16", "P4k_f16", "T4k_bf16_tn", "T4k_bf16_tt", "SK_bf16",
                     "S32_bf16", "S64_f16", "S16_f32", "S16_bf16_kn", "S16_f32_kn", "S64_f32", "S32_f16_tn", "S16_bf16_tt", "D128_bf16"]:
            if name == args.workload:
                continue
            small = pi.WORKLOADS[name].flops < 5e10          # short launches: more of them, or the figure is noise
            r, _ = time_workload(name, max(args.steps, 200) if small else args.steps, args.warmup,
                                 with_torch=not args.no_torch, cpu_seconds=0.0 if args.no_cpu else 1.5)
            log("[bench] %s: %.3f ms  %.1f TFLOP/s  %.0f GB/s  (%s)" % (name, r["event_ms_per_step"], r["tflops_events"],
                                                                        r["gbs_events"], r["plan"]))
            others.append(r)
        out["workloads"] = others
    out["rocm_smi"] = {"before": smi_before, "after": smi_snapshot()}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
