"""Builds libdmi.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SO = os.path.join(HERE, "libdmi.so")
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("dmi_kernels.hip", "dmi_host.hip", "dmi_step.hip",
                                                     "dmi_exporter.hip", "dmi_noalloc.hip")]
HEADERS = [os.path.join(HERE, "csrc", "dmi_internal.h"), os.path.join(HERE, "csrc", "dmi_ring.h"),
           os.path.join(ROOT, "include", "dmi.h"), os.path.join(ROOT, "include", "dmi_debug.h")]


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


TORCH_SO = os.path.join(HERE, "libdmi_torch.so")
TORCH_SRC = os.path.join(HERE, "csrc", "dmi_torch_op.cpp")


def build_torch_op() -> str:
    """The HookPoint operator as a native PyTorch operator (host code only: g++ against libtorch and
    libdmi.so, which must be built first)."""
    import torch
    from torch.utils import cpp_extension as ce
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib")
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
           "-D__HIP_PLATFORM_AMD__=1", "-DUSE_ROCM=1",
           f"-D_GLIBCXX_USE_CXX11_ABI={int(torch._C._GLIBCXX_USE_CXX11_ABI)}",
           "-I", os.path.join(ROOT, "include")]
    for inc in ce.include_paths("cuda"):
        cmd += ["-isystem", inc]
    cmd += [TORCH_SRC, "-o", TORCH_SO, "-L", HERE, "-ldmi", "-L", tlib, "-ltorch", "-ltorch_cpu", "-lc10", "-lc10_hip",
            "-L", os.path.join(rocm, "lib"), "-lamdhip64",
            "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + tlib, "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.check_call(cmd)
    return TORCH_SO


C_CLIENT_SRC = os.path.join(ROOT, "examples", "c_client.c")
C_CLIENT = os.path.join(ROOT, "examples", "c_client")


def build_c_client() -> str:
    """The plain-C example client of the ABI (gcc; links libdmi.so and the HIP runtime)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), C_CLIENT_SRC, "-o", C_CLIENT,
           "-L", HERE, "-ldmi", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2605_11093_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.check_call(cmd)
    return C_CLIENT


if __name__ == "__main__":
    print(build())
    print(build_bench())
    print(build_torch_op())
    print(build_c_client())
