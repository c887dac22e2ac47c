"""The header is C, and a plain C99 program can drive the library's host-only
entry points (no GPU, no C++, no Python in the client)."""
import os
import shutil
import subprocess

import pytest

from paper_1803_09877_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
SRC = os.path.join(ROOT, "tests", "c", "abi_host.c")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_header_is_strict_c99():
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                        "-I", INC, "-x", "c", os.path.join(INC, "draco.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_c_client_runs_against_the_shared_library(tmp_path):
    B.lib()                                               # makes sure the library is built
    libdir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "abi_host")
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", INC, SRC, "-o", exe,
                        "-L", libdir, "-ldraco", "-lm", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
