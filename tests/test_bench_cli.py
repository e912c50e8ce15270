"""Host-side contract of bench.py that needs no GPU: one GPU only, and the product path has no CPU fallback."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""            # no JSON line for a run that did not happen


def test_binding_fails_loudly_without_the_library(tmp_path):
    env = dict(os.environ, LEGEND_HIP_LIB=str(tmp_path / "missing.so"))
    r = subprocess.run([sys.executable, "-c", "import paper_2505_09258_amd.binding"], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "missing" in r.stderr


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_09258_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert "import oracle" not in text and "from oracle" not in text, f
