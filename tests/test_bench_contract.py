"""The benchmark's command line contract: one GPU only, and one JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "alexnet_conv3_n1_f2", "--steps", "20",
                        "--warmup", "5", "--batches", "3"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "whole_layer", "cold", "timing"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["dtype"] == "f32" and d["vs_baseline"] is None
    assert d["config"]["workload"] == "alexnet_conv3_n1_f2" and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "alu") and roof["peak"] in (8000.0, 157.3)
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and 0 < roof["frac"] < 1
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["single_thread"]["cores"] == 1
    # effective FLOP/s definition (Fig. 2 caption): direct-convolution FLOPs over time
    flops = 2 * 1 * 384 * 256 * 13 * 13 * 9
    assert abs(d["value"] - flops / (d["ms_per_step"] * 1e-3) / 1e12) < 0.01 * d["value"]
    assert len(d["timing"]["batch_ms_per_step"]) == 3
