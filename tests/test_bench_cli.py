"""Host-side contract of bench.py that needs no GPU: one GPU only, and the product never imports the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_the_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_02047_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "goose_oracle" not in text and "goose_draft" not in text, f


def test_bench_uses_the_oracle_only_for_the_cpu_baseline():
    text = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    uses = [m.start() for m in re.finditer(r"^\s*(from|import)\s+oracle\b", text, re.M)]
    assert len(uses) == 1 and uses[0] > text.index("def cpu_baseline(")
