"""The boundary is a C ABI: a C99 program that includes include/fcdp.h and
links libfcdp.so builds without warnings and runs its host-only calls."""
import os
import subprocess

import pytest

import paper_2602_06499_amd as fcdp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c99_caller_builds_and_runs(tmp_path):
    lib = fcdp.library_path()
    assert os.path.exists(lib), "build the library first"
    exe = str(tmp_path / "c_abi_check")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe,
                           "-L", os.path.dirname(lib), "-l:libfcdp.so",
                           "-Wl,-rpath," + os.path.dirname(lib) + ":/opt/rocm/lib"])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "c abi ok" in out.stdout


@pytest.mark.gpu
def test_c99_caller_does_gpu_work(tmp_path):
    """The same boundary from C with real device and pinned host memory:
    store, the three fetches, the pageable-memory refusal and a reduce."""
    lib = fcdp.library_path()
    exe = str(tmp_path / "c_abi_gpu")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-unused-parameter",
                           "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                           os.path.join(ROOT, "tests", "c_abi_gpu.c"), "-o", exe,
                           "-L", os.path.dirname(lib), "-l:libfcdp.so", "-L", "/opt/rocm/lib", "-lamdhip64",
                           "-Wl,-rpath," + os.path.dirname(lib) + ":/opt/rocm/lib"])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "c abi gpu ok" in out.stdout
