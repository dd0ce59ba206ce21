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


def test_traffic_figures_in_the_bench_line_are_those_of_the_profile():
    """bench.py prints roofline.traffic from a table, not from counters of its
    own run; the table must be the totals of the counter summary it names."""
    import importlib.util
    import re
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    path = os.path.join(ROOT, bench.TRAFFIC_SOURCE)
    assert os.path.exists(path), "the profile the bench line cites is missing"
    totals = {}
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 9 and cells[0] in bench.MEASURED_TRAFFIC:
            m = re.match(r"\*{0,2}([0-9.]+) MB\*{0,2}$", cells[6])
            if m:
                totals[(cells[0], cells[1])] = float(m.group(1)) * 1e6
    for cfg, (k1, k3f, k3b) in bench.MEASURED_TRAFFIC.items():
        assert totals[(cfg, "K1 unflatten")] == k1, cfg
        assert totals[(cfg, "K3 fp32 -> fp32")] == k3f, cfg
        assert totals[(cfg, "K3 fp32 -> bf16")] == k3b, cfg
