"""Builds tests/native/gpu_native from gpu_native.c: the plain-C program that drives the
library without Python.  Test infrastructure: it links libvccl.so, the C oracle it checks
against, and the HIP runtime."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))


def build_native_check(verbose: bool = True) -> str:
    src = os.path.join(HERE, "gpu_native.c")
    exe = os.path.join(HERE, "gpu_native")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include", src, "-o", exe,
           "-L", os.path.join(ROOT, "paper_2510_00991_amd"), "-lvccl",
           "-L", os.path.join(ROOT, "oracle"), "-lvccl_oracle", "-L", "/opt/rocm/lib", "-lamdhip64",
           # found relative to the program, wherever the tree is copied to
           "-Wl,-rpath,$ORIGIN/../../paper_2510_00991_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.check_call(cmd)
    if verbose:
        print(exe)
    return exe


if __name__ == "__main__":
    build_native_check()
