"""Command-line contracts that need no GPU: the benchmark refuses more than one
GPU with a message, and the product never routes through the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line: nothing was measured


def test_product_does_not_import_the_oracle():
    """Only tests, the smoke check and the benchmark's cpu_baseline leg may use
    the oracle; the package itself must not."""
    pkg = os.path.join(ROOT, "paper_2006_15704_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if not name.endswith((".py", ".hip", ".cpp", ".h")):
                continue
            text = open(os.path.join(dirpath, name)).read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), name
            assert "ddp_oracle" not in text, name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # every use of the oracle sits inside the function of the cpu_baseline leg
    begin = bench.index("def cpu_baseline_leg(")
    end = bench.index("\ndef ", begin + 1)
    uses = [m.start() for m in re.finditer(r"\boracle\.|import oracle", bench)]
    assert uses and all(begin < u < end for u in uses)
    calls = [m.start() for m in re.finditer(r"cpu_baseline_leg\(", bench)]
    guard = bench.index('if "cpu" in legs:')
    assert len(calls) == 2 and max(calls) > guard     # the definition and one guarded call


def test_oracle_does_not_import_the_product():
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", name)).read()
            assert "paper_2006_15704_amd" not in text and "ctypes" not in text
