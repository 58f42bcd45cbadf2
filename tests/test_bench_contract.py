"""Contract checks of bench.py that need no GPU."""
import os
import subprocess
import sys

from tests.conftest import ROOT


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_imports_the_oracle_only_inside_the_cpu_baseline_leg():
    src = open(os.path.join(ROOT, "bench.py")).read()
    lines = [l for l in src.splitlines() if ("import" in l and "oracle" in l)]
    assert lines == ["    from oracle import psd_oracle as orc"] * 2      # cpu_baseline and cpu_baseline_configs
    head = src.split("def layer_work", 1)[0]
    assert "from oracle" not in head and "import oracle" not in head
    extras = open(os.path.join(ROOT, "bench_extras.py")).read()
    assert "oracle" not in extras


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1512_06216_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                text = open(os.path.join(dirpath, f)).read()
                assert "from oracle" not in text and "import oracle" not in text, f
            if f.endswith((".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read(), f
