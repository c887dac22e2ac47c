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
@pytest.mark.parametrize("header", ["draco.h", "draco_bench.h"])
def test_header_is_strict_c99(header):
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                        "-I", INC, "-x", "c", os.path.join(INC, header)], capture_output=True, text=True)
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


@pytest.mark.gpu
@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_c_client_drives_the_three_plan_free_calls_on_the_gpu(tmp_path):
    """encode(assign, grads), decode_repetition(messages, P, s) and decode_cyclic(messages, P, s)
    from a C99 program: no C++, no Python, no plan object on the client's side."""
    B.lib()
    libdir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "abi_gpu")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-unused-parameter", "-I", INC,
                        "-I", "/opt/rocm/include", os.path.join(ROOT, "tests", "c", "abi_gpu.c"), "-o", exe,
                        "-L", libdir, "-ldraco", "-L", "/opt/rocm/lib", "-lamdhip64", "-lm",
                        f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
