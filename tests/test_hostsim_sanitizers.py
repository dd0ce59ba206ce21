"""Host build of the library's own sources under ASan + UBSan (no GPU).

The kernels' index arithmetic and the host code around them are plain C++;
compiled against the stand-in HIP runtime under tests/hostsim/ they run on the
CPU, where an access outside a buffer or undefined behaviour (a misaligned
vector access, a shift or an overflow) is a sanitizer report instead of a GPU
fault.  The driver compares every result with the oracle.  This is a check of
the sources, not a way to run the product: the binding only ever loads
libfcdp.so, and the host build lives in a temporary folder."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SIM = os.path.join(HERE, "hostsim")
CSRC = os.path.join(ROOT, "paper_2602_06499_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"


def _asan_runtime():
    out = subprocess.check_output(
        [CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.fixture(scope="module")
def hostsim_lib(tmp_path_factory):
    if not os.path.exists(CLANG) or _asan_runtime() is None:
        pytest.skip("clang++ with the ASan runtime is not installed")
    so = str(tmp_path_factory.mktemp("hostsim") / "libfcdp_hostsim.so")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fPIC", "-shared",
           "-I", SIM, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "c++",
           os.path.join(SIM, "globals.cpp"), os.path.join(CSRC, "fcdp_layout.cpp"),
           os.path.join(CSRC, "fcdp_kernels.hip"), os.path.join(CSRC, "fcdp_api.hip"),
           "-o", so]
    subprocess.check_call(cmd)
    return so


def _run(so, *extra):
    env = dict(os.environ)
    pre = [_asan_runtime()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    return subprocess.run([sys.executable, "-u", os.path.join(SIM, "driver.py"), so, *extra],
                          env=env, capture_output=True, text=True, timeout=600)


def test_entry_points_clean_under_sanitizers(hostsim_lib):
    r = _run(hostsim_lib)
    tail = (r.stdout[-1500:] + "\n" + r.stderr[-4000:])
    assert r.returncode == 0, tail
    assert "hostsim ok" in r.stdout, tail
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail


def test_sanitizers_see_a_planted_overrun(hostsim_lib):
    """A buffer 2 bytes short (the mistake is planted in the caller, on the
    CPU) must end the run with an ASan report."""
    r = _run(hostsim_lib, "--plant-short-output")
    assert r.returncode != 0
    assert "AddressSanitizer" in r.stderr and "heap-buffer-overflow" in r.stderr
    assert "went unseen" not in r.stdout


def test_two_threads_under_thread_sanitizer(tmp_path):
    """The header allows data calls from several threads as long as they do
    not share a staging buffer, a cache state or the timing pool.  Two threads
    hammer the fetch paths, the reduce and the link counters of the host build
    under ThreadSanitizer: no race report, right bytes, no lost counter update."""
    tsan = subprocess.run([CLANG, "-print-file-name=libclang_rt.tsan-x86_64.a"],
                          capture_output=True, text=True).stdout.strip()
    if not os.path.exists(CLANG) or not (os.path.isabs(tsan) and os.path.exists(tsan)):
        pytest.skip("clang++ with the TSan runtime is not installed")
    exe = str(tmp_path / "fcdp_threads")
    subprocess.check_call([CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-fPIE", "-pie",
                           "-I", SIM, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "c++",
                           os.path.join(SIM, "globals.cpp"), os.path.join(CSRC, "fcdp_layout.cpp"),
                           os.path.join(CSRC, "fcdp_kernels.hip"), os.path.join(CSRC, "fcdp_api.hip"),
                           os.path.join(SIM, "threads.cpp"), "-o", exe, "-lpthread"])
    env = dict(os.environ)
    env["TSAN_OPTIONS"] = "halt_on_error=0:report_signal_unsafe=0"
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    tail = r.stdout[-1500:] + "\n" + r.stderr[-4000:]
    assert "ThreadSanitizer" not in r.stderr, tail
    assert r.returncode == 0 and "threads ok" in r.stdout, tail
