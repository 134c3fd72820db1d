"""Builds tests/c_abi/c_abi_check (plain C against include/wkv6.h, the HIP runtime and the C
oracle); called from __graft_entry__.build().  The binary travels with the tree to the GPU machine,
where tests/test_gpu_c_abi.py runs it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BINARY = os.path.join(HERE, "c_abi_check")


def build_c_abi_check():
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    pkg = os.path.join(ROOT, "paper_2407_12077_amd")
    cmd = ["gcc", "-O2", "-std=c11", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-o", BINARY, os.path.join(HERE, "c_abi_check.c"),
           "-L", pkg, "-L", os.path.join(ROOT, "oracle"), "-L", os.path.join(rocm, "lib"),
           "-lwkv6", "-lwkv6_oracle", "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2407_12077_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.check_call(cmd)
    return BINARY


if __name__ == "__main__":
    print(build_c_abi_check())
