"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the code that runs on the host: the
CPU oracle and the library's planner with its selector-table parser, each built with the host
compiler and driven by a small program under tests/sanitize/.  (The GPU side has no sanitizer
on this kind of machine; these are the paper's "extended validators" of Section 3.3 for the
part of the library a sanitizer can see.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", PEAK_GEMM_TUNING="")
ENV.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the library list


def _build_and_run(cmd, exe, args, tmp_path):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe] + args, capture_output=True, text=True, timeout=300, env=ENV, cwd=str(tmp_path))
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    return r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host C compiler")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    out = _build_and_run(["gcc", "-std=c11"] + SAN + [os.path.join(ROOT, "oracle", "oracle_gemm.c"),
                                                      os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"),
                                                      "-o", exe, "-lm", "-lpthread"], exe, [], tmp_path)
    assert "oracle sanitizer run clean" in out


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_planner_and_table_parser_under_sanitizers(tmp_path):
    exe = str(tmp_path / "planner_san")
    out = _build_and_run(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                         [os.path.join(ROOT, "paper_2512_19018_amd", "csrc", "planner.cpp"),
                          os.path.join(ROOT, "tests", "sanitize", "planner_main.cpp"), "-o", exe, "-ldl"],
                         exe, [str(tmp_path)], tmp_path)
    assert "planner sanitizer run clean" in out
