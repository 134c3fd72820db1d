"""Host-side sanitizer runs (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only; the GPU code
objects are built as usual and never run here).

* the C oracles with a plain-C driver that walks their threaded, single-threaded, empty and
  bad-argument paths (``tests/sanitize/oracle_check.c``);
* the library's C ABI: its sources compiled by hipcc with the sanitizers on the host side and a
  driver that calls every validation path (``tests/sanitize/boundary_check.cpp``); every call is
  rejected before a launch, so no GPU is needed.

Commands:
  gcc -std=c11 -g -O1 -fsanitize=address,undefined -fno-sanitize-recover=all -pthread \
      tests/sanitize/oracle_check.c oracle/*.c -lm
  hipcc --offload-arch=gfx950 -O1 -g -std=c++17 -Xarch_host -fsanitize=address \
      -Xarch_host -fsanitize=undefined -Xarch_host -fno-sanitize-recover=all ... \
      tests/sanitize/boundary_check.cpp paper_2407_12077_amd/csrc/*.hip
"""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_check"
    srcs = [os.path.join(ROOT, "tests", "sanitize", "oracle_check.c")] + sorted(glob.glob(os.path.join(ROOT, "oracle", "*.c")))
    subprocess.check_call(["gcc", "-std=c11", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-pthread", "-o", str(exe)] + srcs + ["-lm"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr


def test_boundary_validation_under_asan_and_ubsan(tmp_path):
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not on PATH")
    exe = tmp_path / "boundary_check"
    csrc = os.path.join(ROOT, "paper_2407_12077_amd", "csrc")
    srcs = [os.path.join(ROOT, "tests", "sanitize", "boundary_check.cpp")] + sorted(glob.glob(os.path.join(csrc, "*.hip")))
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-o", str(exe)] + srcs
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    # the HIP runtime keeps process-lifetime allocations of its own: leak checking is for the oracle run
    env = dict(ENV, ASAN_OPTIONS="detect_leaks=0")
    out = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr
