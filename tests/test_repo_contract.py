"""Repository-level contracts: the product never touches the oracle, and bench.py's JSON line."""
import json
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_product_path_never_imports_or_links_the_oracle():
    pkg = os.path.join(ROOT, "paper_2408_04093_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"\boracle\b", text), f"{f} mentions the oracle"
    for f in ("ta_oracle.c", "ta_oracle.py"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2408_04093_amd" not in text and "tree_attn.h" not in text


def test_workload_generators_hold_no_arithmetic_of_the_method():
    text = open(os.path.join(ROOT, "ta_workloads.py")).read()
    assert "import oracle" not in text and "paper_2408_04093_amd" not in text
    assert not re.search(r"softmax|logsumexp|\.exp\(", text)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2", "--no-extra"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    rec = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
              "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in rec, k
    assert rec["n_gpus"] == 1 and rec["steps"] == 5 and rec["unit"] == "GB/s" and rec["data"] == "synthetic"
    assert rec["config"]["workload"] == "llama128k" and rec["vs_baseline"] is None
    rf = rec["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rec["cpu_baseline"]["kind"] == "oracle" and rec["cpu_baseline"]["cores"] >= 1
    assert rec["parity_vs_oracle"]["lse_abs"] <= 1e-4
