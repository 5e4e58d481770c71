"""Build libmerit.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libmerit.so")

SOURCES = ["merit_plan.cpp", "pool2d.hip", "sad_search.hip", "conv2d.hip", "conv2d_chws.hip", "corr.hip", "dwconv.hip", "sepfilter.hip", "bilateral.hip", "probe.hip"]
HEADERS = [os.path.join(CSRC, "merit_internal.h"), os.path.join(ROOT, "include", "merit.h"),
           os.path.join(ROOT, "include", "merit_probe.h")]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the MERIT HIP library cannot be built")


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 into one shared library."""
    if not force and not is_stale():
        return LIB_PATH
    common = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              # keep hipcc from forming packed-fp32 VALU ops
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wall", "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra_flags]
    # one object per source, compiled side by side (the convolution file dominates), then one link
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.splitext(s)[0] + ".o") for s in SOURCES]

    def compile_one(job):
        src, obj = job
        return subprocess.run(common + ["-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        for proc in pool.map(compile_one, zip(SOURCES, objs)):
            if proc.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    proc = subprocess.run(common + ["-shared", "-o", LIB_PATH] + objs, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc (link) failed:\n" + proc.stdout + proc.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library())
