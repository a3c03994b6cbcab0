"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_never_reaches_the_oracle_outside_its_cpu_baseline_leg():
    src = open(os.path.join(ROOT, "bench.py")).read()
    body = src.split("def cpu_baseline", 1)[1].split("\ndef ", 1)[0]
    assert "from oracle import" in body
    assert src.count("oracle import") == 1, "the oracle may only be imported inside cpu_baseline"
    pkg = os.path.join(ROOT, "paper_2312_11514_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            assert "oracle" not in open(os.path.join(pkg, name)).read(), name
    for name in os.listdir(os.path.join(ROOT, "workloads")):
        if name.endswith(".py"):
            text = open(os.path.join(ROOT, "workloads", name)).read()
            assert "import oracle" not in text and "from oracle" not in text, name
