"""Streaming microbenchmark (tests/stream_probe/stream_probe.hip): kernels that move the benchmark
workload's bytes with no arithmetic, one workgroup per compute unit.  Its figures are the
rate the memory system delivers to this access pattern, the reference beside which the kernel's
time is read; the test prints them and checks only that they are sane (every variant between 1 and 8 TB/s, the contiguous variant
not slower than the strided one by more than noise)."""
import os
import re
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
BINARY = os.path.join(HERE, "stream_probe", "stream_probe")


def test_stream_probe_rates(gpu_device):
    if not os.path.exists(BINARY):
        pytest.fail(f"{BINARY} is missing: run __graft_entry__.build() first")
    out = subprocess.run([BINARY, "30"], capture_output=True, text=True, timeout=100)
    print(out.stdout, flush=True)
    assert out.returncode == 0, out.stdout + out.stderr
    rates = {}
    for line in out.stdout.splitlines():
        m = re.match(r"(.*?)\s+([\d.]+) us\s+([\d.]+) TB/s", line)
        if m:
            rates[m.group(1).strip()] = float(m.group(3))
    assert len(rates) == 10
    assert all(1.0 < v < 8.0 for v in rates.values()), rates
    strided = rates["kernel layout (128 B rows), nt loads, write-through stores"]
    slabs = rates["contiguous slabs, nt loads, write-through stores"]
    assert slabs > 0.9 * strided
