"""Builds libdmi.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SO = os.path.join(HERE, "libdmi.so")
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("dmi_kernels.hip", "dmi_host.hip")]
HEADERS = [os.path.join(HERE, "csrc", "dmi_internal.h"), os.path.join(ROOT, "include", "dmi.h")]


def hipcc() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


BENCH_SO = os.path.join(HERE, "libdmi_bench.so")
BENCH_SRC = os.path.join(HERE, "csrc", "bench_kernels.hip")


def build_bench() -> str:
    """Harness-side kernels for bench.py (sleep, streaming GEMV)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I", os.path.join(ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           BENCH_SRC, "-o", BENCH_SO]
    subprocess.check_call(cmd)
    return BENCH_SO


def build(force: bool = True) -> str:
    if not force and os.path.exists(SO):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(SO) >= newest:
            return SO
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I", os.path.join(ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           *SOURCES, "-o", SO, "-lpthread"]
    subprocess.check_call(cmd)
    return SO


if __name__ == "__main__":
    print(build())
    print(build_bench())
