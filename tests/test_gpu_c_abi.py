"""The boundary used from plain C (no Python, no torch): compiled with gcc and run as a child process."""
import os
import subprocess
import sys

import pytest

import paper_2507_13522_amd as sh
from paper_2507_13522_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_abi", "abi_smoke.c")


def compile_smoke(out: str) -> None:
    sh.lib()                                  # makes sure the library exists
    libdir = os.path.dirname(build.LIB)
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I" + os.path.join(ROOT, "include"), SRC, "-o", out, "-L" + libdir, "-lshadow",
                           "-L/opt/rocm/lib", "-lamdhip64", "-lm", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])


def test_c_program_compiles_against_the_header(tmp_path):
    compile_smoke(str(tmp_path / "abi_smoke"))


@pytest.mark.gpu
def test_c_program_runs(tmp_path):
    exe = str(tmp_path / "abi_smoke")
    compile_smoke(exe)
    print("case c abi", flush=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, r.stdout + r.stderr
