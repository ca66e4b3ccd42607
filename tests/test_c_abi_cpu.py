"""The boundary from plain C: include/vccl.h must compile as C11 (and as C++17) with
warnings as errors, and a C program linked against libvccl.so must be able to use the
host-only entry points without a device."""
import os
import subprocess

import pytest

import paper_2510_00991_amd as vccl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
SRC = os.path.join(ROOT, "tests", "native", "abi_check.c")


def test_header_is_valid_c_and_cxx(tmp_path):
    for compiler, std, name in (("gcc", "-std=c11", "h.c"), ("g++", "-std=c++17", "h.cpp")):
        f = tmp_path / name
        f.write_text('#include "vccl.h"\nint main(void) { return VCCL_OK; }\n')
        subprocess.check_call([compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", INC,
                               "-c", str(f), "-o", str(tmp_path / (name + ".o"))])


def test_c_program_uses_the_host_only_entry_points(tmp_path):
    lib = vccl.lib_path()
    if not os.path.exists(lib):
        pytest.fail("libvccl.so has not been built")
    exe = tmp_path / "abi_check"
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", INC, SRC,
                           "-o", str(exe), "-L", os.path.dirname(lib), "-lvccl",
                           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib"])
    rv = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert rv.returncode == 0, rv.stdout + rv.stderr
    assert "abi ok" in rv.stdout
