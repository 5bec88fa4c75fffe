"""The parts of bench.py's contract that need no GPU: more than one GPU is refused with a message, and the product
path never imports the oracle (only tests, the smoke check and the benchmark's CPU-baseline leg may)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_the_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2112_00709_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), f
                assert "fb_oracle" not in text and "viterbi_oracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # in the benchmark the oracle is imported inside the CPU-baseline branch only
    assert len(re.findall(r"^\s*import oracle\b", bench, re.M)) == 1
    assert bench.index("if not args.no_cpu_baseline:") < bench.index("import oracle")
