"""The C ABI from plain C: runs the prebuilt tests/c_abi/c_abi_check (no Python or PyTorch in
that process), which calls two entry points on device 0 and compares with the fp64 oracle."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
BINARY = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_abi_check")


def test_c_program_calls_the_library(gpu_device):
    if not os.path.exists(BINARY):                 # normally built beforehand by build(); gcc only, seconds
        sys.path.insert(0, os.path.dirname(BINARY))
        from build_check import build_c_abi_check
        build_c_abi_check()
    done = subprocess.run([BINARY], capture_output=True, text=True, timeout=110)
    print(done.stdout, done.stderr, flush=True)
    assert done.returncode == 0, (done.returncode, done.stderr)
    assert "err_out" in done.stdout
