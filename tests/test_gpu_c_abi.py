"""The boundary from plain C: tests/c_abi/c_abi_check.c (hipMalloc'd buffers, the five calls, comparison with
the oracle's C functions, no Python or torch in that process) is compiled with gcc and run."""
import os
import subprocess

import pytest

import oracle
from paper_2402_02320_amd import spin

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_abi", "c_abi_check.c")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def compile_cmd(out, syntax_only=False):
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROCM, "include"), SRC]
    if syntax_only:
        return cmd + ["-fsyntax-only"]
    libdirs = [os.path.dirname(spin.LIB_PATH), os.path.join(ROOT, "oracle"), os.path.join(ROCM, "lib")]
    for d in libdirs:
        cmd += ["-L", d, "-Wl,-rpath," + d]
    return cmd + ["-lspin", "-loracle", "-lamdhip64", "-o", out]


def test_header_is_valid_c_and_cxx():
    for name in ("spin.h", "spin_bench.h"):
        hdr = os.path.join(ROOT, "include", name)
        subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
        subprocess.run(["g++", "-std=c++11", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr],
                       check=True)


def test_c_harness_compiles():
    subprocess.run(compile_cmd(None, syntax_only=True), check=True)


@pytest.mark.gpu
def test_c_program_matches_the_oracle(tmp_path):
    oracle.lib()                                           # makes sure liboracle.so is built
    exe = str(tmp_path / "c_abi_check")
    subprocess.run(compile_cmd(exe), check=True)
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    assert res.returncode == 0 and "c abi ok" in res.stdout, res.stdout
