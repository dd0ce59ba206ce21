"""What bench.py and the entry file promise that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args],
                          capture_output=True, text=True, timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be taken for a result


def test_no_gpu_is_a_loud_failure_not_a_cpu_run():
    import torch
    if torch.cuda.is_available():
        return
    r = _bench("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "needs a GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_entry_file_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g
    assert callable(g.build) and callable(g.smoke)


def test_product_never_imports_the_oracle():
    """Only tests, smoke() and the cpu_baseline leg of bench.py may touch oracle/."""
    pkg = os.path.join(ROOT, "paper_2602_06499_amd")
    for dirpath, _dirs, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "fcdp_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    head, _, tail = bench.partition("if not args.no_cpu_baseline:")
    assert "import oracle" not in head, "bench.py may import the oracle only in its cpu_baseline leg"
    assert "import oracle" in tail
