"""Contracts that need no GPU: the benchmark refuses more than one GPU, the product path has no CPU fallback,
and nothing outside tests / smoke / the benchmark's CPU-baseline leg touches the oracle."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert p.returncode != 0 and "one GPU" in (p.stderr + p.stdout)


def test_product_path_has_no_cpu_fallback():
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2304_07741_amd import harness, workloads as wl

    with pytest.raises(RuntimeError, match="no CPU path"):
        harness.DagRunner(wl.blob_shift_residual(64), (1, 64, 8, 8), "bf16")


def test_only_tests_smoke_and_the_cpu_baseline_use_the_oracle():
    """The package never imports the oracle; bench.py does so only inside cpu_baseline; the entry file only in smoke."""
    pkg = os.path.join(ROOT, "paper_2304_07741_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b|canvas_oracle\.|solver_oracle", text, re.M), f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    body = bench[bench.index("def cpu_baseline"):bench.index("def main")]
    assert "from oracle import" in body and "oracle" not in bench.replace(body, "").replace("the oracle", "").replace('"oracle"', "").replace("CPU oracle", "")
    entry = open(os.path.join(ROOT, "__graft_entry__.py")).read()
    smoke = entry[entry.index("def smoke"):]
    assert "oracle" in smoke
