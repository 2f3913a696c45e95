"""Compile the HIP library for gfx950 into paper_2512_19018_amd/libpeak_gemm.so.

The kernel variants are spread over several translation units (csrc/variants_*.hip)
that compile in parallel into csrc/_build/*.o; peak_gemm.hip holds the C ABI, the
selector and the small kernels.
"""
import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
OUT = os.path.join(HERE, "libpeak_gemm.so")
HEADERS = [os.path.join(CSRC, h) for h in ("gemm_device.h", "gemm16_device.h", "skinny_device.h", "variant.h", "variant16.h", "planner.h",
                                           "variants_16nt.inc", "variants_16nn.inc")]
HEADERS.append(os.path.join(HERE, "..", "include", "peak_gemm.h"))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 VALU ops
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
    "-Wno-inline-asm",                                               # m0 named as clobbered by the hand-issued loads
]


def sources():
    # the kernels' translation units and the host-only planner (plain C++, compiled by the same driver)
    return sorted(glob.glob(os.path.join(CSRC, "*.hip"))) + [os.path.join(CSRC, "planner.cpp")]


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _obj_of(src):
    return os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, extra):
    subprocess.check_call([_hipcc()] + HIPCC_FLAGS + list(extra) + ["-c", src, "-o", _obj_of(src)])
    return src


def build(force: bool = True, extra=(), jobs=None) -> str:
    """force=True recompiles every translation unit; otherwise only those older
    than their source, the shared headers or this script."""
    os.makedirs(OBJ, exist_ok=True)
    common = HEADERS + [os.path.abspath(__file__)]
    todo = [s for s in sources() if force or _stale(_obj_of(s), [s] + common)]
    if todo:
        jobs = jobs or min(len(todo), max(1, min(16, os.cpu_count() or 1)))
        with concurrent.futures.ThreadPoolExecutor(jobs) as pool:
            for done in pool.map(lambda s: _compile(s, extra), todo):
                print("compiled", os.path.basename(done), flush=True)
    objs = [_obj_of(s) for s in sources()]
    if todo or _stale(OUT, objs):
        subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs + ["-ldl"])
    return OUT


if __name__ == "__main__":
    args = sys.argv[1:]
    incremental = "--incremental" in args
    print(build(force=not incremental, extra=[a for a in args if a != "--incremental"]))
