"""Correctness validator over sampled kernel settings, without a second implementation.

The paper's "correctness validators" (Section 3.3) take a kernel context and a
budget of execution-parameter settings to sample; the portable task compares
outputs against a trusted reference within a tolerance, and the extended tasks
look for what output comparison misses: memory-safety violations and
nondeterminism.  This module is that task for the library's own kernels, for
use on a GPU machine where no sanitizer is at hand:

  * reference: the plainest kernel variant that accepts the problem (register
    staging, 64x64 tiles, no K split) plays the paper's "simple trusted kernel";
    every sampled setting must agree with it within the dtype's tolerance;
  * canaries: A, B, C and the workspace sit inside larger allocations whose
    guard bands hold a NaN pattern; after each run the bands of C and of the
    workspace, and the padding columns of C beyond N, must be byte-identical
    (stray writes), and the result must be finite (a stray read of a band of A
    or B that reaches an accumulator shows as NaN);
  * with beta == 0, C starts as NaN and must come back finite (C is write-only);
  * determinism: every setting runs twice and must give the same bits.

    python -m paper_2512_19018_amd.validate --shape bf16:0:1:300:520:1000 --samples 24

Needs a GPU; torch is used for device memory and comparisons only.  The CPU
oracle of the test suite is deliberately not used here.
"""
from __future__ import annotations

import argparse
import sys

from . import binding as pg
from .tune import DT_NAMES, candidates

GUARD_BYTES = 4096
TOL = {pg.PEAK_DT_F32: 1e-5, pg.PEAK_DT_F16: 2e-2, pg.PEAK_DT_BF16: 2e-2}     # relative Frobenius
_NAN16 = {pg.PEAK_DT_F16: 0x7E01, pg.PEAK_DT_BF16: 0x7FC1}


def sample_settings(cands, samples, seed=0):
    """At most `samples` of the accepted (variant id, name, split, info) settings:
    all of them if they fit the budget, else a seeded choice without repetition
    (a linear congruential walk, so the choice does not depend on any library)."""
    cands = list(cands)
    if samples is None or samples >= len(cands):
        return cands
    picked, state, left = [], (seed * 2654435761 + 12345) & 0xFFFFFFFF, list(range(len(cands)))
    for _ in range(max(samples, 0)):
        state = (state * 1664525 + 1013904223) & 0xFFFFFFFF
        picked.append(left.pop(state % len(left)))
    return [cands[i] for i in sorted(picked)]


def reference_setting(cands):
    """The plainest accepted setting: register-staged 64x64 tiles if present, else
    the first register-staged one, else the first of all; always without a K split."""
    unsplit = [c for c in cands if c[2] == 1] or list(cands)
    for key in ("_r64x64_", "_r128x128_"):
        for c in unsplit:
            if key in c[1]:
                return c
    return unsplit[0]


class _Guarded:
    """rows x ld elements of `tdt` between two guard bands of NaN bytes."""

    def __init__(self, torch, rows, ld, tdt, dtype, fill, device="cuda"):
        self.torch, self.es = torch, torch.empty((), dtype=tdt).element_size()
        self.n = max(rows * ld, 1)
        g = GUARD_BYTES // self.es
        self.g = g
        self.buf = torch.empty(self.n + 2 * g, dtype=tdt, device=device)
        self._poison(self.buf, dtype)
        self.body = self.buf[g:g + self.n]
        if fill is not None:
            self.body[:rows * ld].view(rows, ld).copy_(fill)
        self.before = self.buf[:g].clone()
        self.after = self.buf[g + self.n:].clone()

    @staticmethod
    def _poison(t, dtype):
        import torch
        if dtype == pg.PEAK_DT_F32:
            t.fill_(float("nan"))
        else:
            t.view(torch.int16).fill_(_signed(_NAN16[dtype]))

    def ptr(self):
        return self.body.data_ptr()

    def guards_intact(self):
        t = self.torch
        b = t.equal(self.buf[:self.g].view(t.uint8), self.before.view(t.uint8))
        a = t.equal(self.buf[self.g + self.n:].view(t.uint8), self.after.view(t.uint8))
        return bool(a and b)


def _signed(u16):
    return u16 - 65536 if u16 >= 32768 else u16


def validate(dtype, transA, transB, M, N, K, alpha=1.0, beta=0.0, samples=None, seed=0, ldc_pad=8, log=None):
    """Runs the checks above over the sampled settings.  Returns a list of
    (setting name, split, problem text) for every failed check; empty = clean."""
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("validate needs a GPU")
    tdt = {pg.PEAK_DT_F32: torch.float32, pg.PEAK_DT_F16: torch.float16, pg.PEAK_DT_BF16: torch.bfloat16}[dtype]
    gen = torch.Generator(device="cuda").manual_seed(1234 + seed)
    scale = 1.0 / max(K, 1) ** 0.5
    a_rows, a_ld = (K, M) if transA else (M, K)
    b_rows, b_ld = (N, K) if transB else (K, N)
    ldc = N + ldc_pad
    hA = (torch.randn((a_rows, a_ld), device="cuda", generator=gen) * scale).to(tdt)
    hB = torch.randn((b_rows, b_ld), device="cuda", generator=gen).to(tdt)
    hC = torch.randn((M, ldc), device="cuda", generator=gen).to(tdt)
    A = _Guarded(torch, a_rows, a_ld, tdt, dtype, hA)
    B = _Guarded(torch, b_rows, b_ld, tdt, dtype, hB)
    stream = torch.cuda.current_stream().cuda_stream

    cands = candidates(dtype, transA, transB, M, N, K, ldc=ldc)
    if not cands:
        return [("-", 0, "no kernel variant accepts the problem")]
    ref_set = reference_setting(cands)
    chosen = sample_settings(cands, samples, seed)
    if ref_set not in chosen:
        chosen = [ref_set] + chosen
    failures, ref_vals = [], None

    def run_once(vid, split):
        C = _Guarded(torch, M, ldc, tdt, dtype, hC if beta != 0.0 else None)     # beta == 0: C starts as NaN
        pad0 = C.body.view(M, ldc)[:, N:].clone()
        with pg.Plan(M, N, K, dtype, transA, transB, a_ld, b_ld, ldc, pg.force_flags(vid, split)) as plan:
            wsb = plan.workspace_bytes
            W = _Guarded(torch, 1, max(wsb // 4, 64), torch.float32, pg.PEAK_DT_F32, None)
            # the workspace must be 256-byte aligned: the guard band is a multiple of that
            plan.run(alpha, A.ptr(), B.ptr(), beta, C.ptr(), W.ptr(), wsb, stream)
            torch.cuda.synchronize()
        problems = []
        if not C.guards_intact():
            problems.append("wrote outside C")
        if not W.guards_intact():
            problems.append("wrote outside the workspace")
        if not torch.equal(C.body.view(M, ldc)[:, N:].view(torch.uint8), pad0.view(torch.uint8)):
            problems.append("wrote into the padding columns of C")
        out = C.body.view(M, ldc)[:, :N].clone()
        if not bool(torch.isfinite(out.float()).all()):
            problems.append("non-finite result (read of a guard band, or of C with beta == 0)")
        return out, problems

    # the reference first
    order = [ref_set] + [c for c in chosen if c != ref_set]
    for vid, name, split, info in order:
        out1, problems = run_once(vid, split)
        out2, _ = run_once(vid, split)
        if not torch.equal(out1.view(torch.uint8), out2.view(torch.uint8)):
            problems.append("two runs differ")
        if ref_vals is None:
            ref_vals = out1.double()
        else:
            num = float(torch.linalg.norm(out1.double() - ref_vals))
            den = float(torch.linalg.norm(ref_vals))
            err = num / den if den > 0 else (0.0 if num == 0 else float("inf"))
            # both sides carry the dtype's rounding, hence twice the tolerance of one
            if not err <= 2 * TOL[dtype]:
                problems.append("disagrees with %s: relative error %.3e" % (ref_set[1], err))
        if log:
            log("  %-32s split=%-3d %s" % (name, split, "ok" if not problems else "; ".join(problems)))
        failures += [(name, split, p) for p in problems]
    if not (A.guards_intact() and B.guards_intact()):
        failures.append(("-", 0, "an input's guard band changed"))
    return failures


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--shape", action="append", default=[], metavar="DT:TA:TB:M:N:K", required=True)
    ap.add_argument("--samples", type=int, default=None, help="settings to sample per shape (default: all)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--beta", type=float, default=0.0)
    args = ap.parse_args(argv)
    bad = 0
    for s in args.shape:
        dt, ta, tb, M, N, K = s.split(":")
        print("%s transA=%s transB=%s %sx%sx%s" % (dt, ta, tb, M, N, K), file=sys.stderr, flush=True)
        f = validate(DT_NAMES[dt], int(ta), int(tb), int(M), int(N), int(K), 1.0, args.beta, args.samples, args.seed,
                     log=lambda m: print(m, file=sys.stderr, flush=True))
        bad += len(f)
    print("%d problem(s)" % bad)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
