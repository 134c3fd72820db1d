"""Builds tests/stream_probe/stream_probe for gfx950; called from __graft_entry__.build().  The binary
travels with the tree to the GPU machine, where tests/test_gpu_stream_probe.py runs it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
BINARY = os.path.join(HERE, "stream_probe")


def build_stream_probe():
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-o", BINARY, os.path.join(HERE, "stream_probe.hip")]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    return BINARY


if __name__ == "__main__":
    print(build_stream_probe())
