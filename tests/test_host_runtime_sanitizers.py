"""The library's host runtime (rings, admission, commit discovery, drain thread, exporter, replayable
steps: csrc/dmi_host.hip, dmi_step.hip, dmi_exporter.hip) under ThreadSanitizer and AddressSanitizer,
on the CPU.  The three files are compiled as plain C++ against a stand-in for the HIP runtime
(tests/cpu_runtime/), with a CPU executor behind the kernel-launch seam in place of the device code,
and driven by tests/cpu_runtime/driver.cpp from five kinds of threads at once (producer, the
library's drain thread, consumer or exporter, a statistics reader, a thread issuing drains)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CPU = os.path.join(ROOT, "tests", "cpu_runtime")
CSRC = os.path.join(ROOT, "paper_2605_11093_amd", "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("dmi_host.hip", "dmi_step.hip", "dmi_exporter.hip")] + \
          [os.path.join(CPU, f) for f in ("fake_hip.cpp", "cpu_kernels.cpp", "driver.cpp")]


def _build(tmp_path, sanitizer):
    exe = str(tmp_path / f"driver_{sanitizer}")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", f"-fsanitize={sanitizer}", "-pthread",
           "-I", CPU, "-I", CSRC, "-I", os.path.join(ROOT, "include"), "-o", exe]
    for src in SOURCES:
        cmd += ["-x", "c++", src]
    subprocess.check_call(cmd)
    return exe


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
@pytest.mark.parametrize("sanitizer,iters", [("thread", 3000), ("address", 3000)])
def test_host_runtime_is_clean_under(tmp_path, sanitizer, iters):
    exe = _build(tmp_path, sanitizer)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66 second_deadlock_stack=1",
               ASAN_OPTIONS="detect_leaks=1 exitcode=67")
    p = subprocess.run([exe, str(iters)], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=280)
    out = p.stdout.decode(errors="replace")
    assert p.returncode == 0, out[-6000:]
    assert "all scenarios passed" in out
