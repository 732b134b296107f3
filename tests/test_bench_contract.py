"""bench.py keeps its one-line JSON contract (checked on a small workload so the test takes seconds)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [["--workload", "encoder_d768"], ["--workload", "mlp_784_1024_1024_10"],
                                   ["--workload", "encoder_d768", "--mode", "two_level"],
                                   ["--workload", "encoder_d768", "--mode", "sequential"],
                                   ["--workload", "encoder_d768", "--mode", "backprop"]])
def test_bench_prints_one_json_line_with_the_contract_keys(gpu, extra):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "3", "--warmup", "1"] + extra,
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["data"] == "synthetic" and "workload" in d["config"] and d["value"] > 0 and d["ms_per_step"] > 0
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["peak"] > 0 and 0 < roof["frac"] < 1.0
    assert abs(roof["achieved"] / roof["peak"] - roof["frac"]) < 1e-9 and "traffic" in roof
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
