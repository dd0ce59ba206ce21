"""The oracle's C source under ASan + UBSan: the pin tests are run in a child
process against a sanitized build, so an index that leaves a buffer or an
undefined operation inside the oracle is a report, not a silently wrong
expected value."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "fcdp_oracle.c")

CHILD = r"""
import ctypes, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import numpy as np
import oracle
lib = ctypes.CDLL(sys.argv[1])
lib.fcdp_oracle_segments.restype = ctypes.c_int64
lib.fcdp_oracle_bf16_rne.restype = ctypes.c_uint16
lib.fcdp_oracle_bf16_rne.argtypes = [ctypes.c_float]
oracle._lib = lib
if len(sys.argv) > 2:       # a caller's mistake on purpose: the output is one shard short
    shards = [np.arange(64, dtype=np.uint16) for _ in range(4)]
    H = np.empty(3 * 64, dtype=np.uint16)
    ptrs = (ctypes.c_void_p * 4)(*[s.ctypes.data for s in shards])
    lib.fcdp_oracle_cache_store(ptrs, ctypes.c_int64(64), ctypes.c_int32(4), ctypes.c_int32(2),
                                ctypes.c_void_p(H.ctypes.data))
    print("went unseen")
    sys.exit(0)
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider",
                      {tests!r} + "/test_oracle_pins.py", {tests!r} + "/test_alg1_oracle.py"]))
"""


def _libasan():
    out = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    if _libasan() is None:
        pytest.skip("gcc's ASan runtime is not installed")
    d = tmp_path_factory.mktemp("oracle_asan")
    so = str(d / "liboracle_asan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-shared", "-fPIC", "-o", so, SRC])
    child = str(d / "child.py")
    with open(child, "w") as f:
        f.write(CHILD.format(root=ROOT, tests=HERE))
    return so, child


def _run(so, child, *extra):
    env = dict(os.environ)
    pre = [_libasan()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"
    return subprocess.run([sys.executable, "-u", child, so, *extra], env=env,
                          capture_output=True, text=True, timeout=900)


def test_pins_pass_on_the_sanitized_oracle(sanitized):
    r = _run(*sanitized)
    tail = r.stdout[-2000:] + "\n" + r.stderr[-3000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail


def test_sanitized_oracle_reports_a_planted_overrun(sanitized):
    r = _run(*sanitized, "--plant")
    assert r.returncode != 0
    assert "AddressSanitizer" in r.stderr
    assert "went unseen" not in r.stdout
