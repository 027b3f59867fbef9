"""The benchmark's own contract, on the GPU: one JSON line with the agreed fields, for the smallest configuration."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines                       # exactly one JSON line on stdout
    return json.loads(lines[0])


def test_bench_line_of_the_tiny_configuration():
    print("bench.py --config tiny", flush=True)
    d = _run("--config", "tiny", "--tokens", "16", "--steps", "5", "--warmup", "2", "--sweep-iters", "2")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["higher_is_better"] is False
    assert d["unit"] == "us/batch" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert abs(d["value"] - d["ms_per_step"] * 1e3) < 0.02 and d["value"] > 0
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3 and 0 < rf["frac"] < 1
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["unit"] == d["unit"] and cb["sample"]
    for name in ("fp8_weights",):                        # (H = 512, F = 1024: multiples of 128 as well)
        assert d[name]["us_per_batch"] > 0
    assert d["mxfp4_weights"]["us_per_batch"] > 0
    assert {r["remap"] for r in d["sweep"]} == {"off", "moderate", "aggressive"}


def test_bench_stack_mode():
    print("bench.py --config tiny --stack 3", flush=True)
    d = _run("--config", "tiny", "--tokens", "16", "--stack", "3", "--steps", "3", "--warmup", "1",
             "--layer-policy", "0:off,2:moderate")
    assert set(d["stack"]) == {"off", "aggressive", "layer_policy"}
    for v in d["stack"].values():
        assert v["us_graph_median"] > 0 and v["us_eager_median"] > 0
    assert d["stack"]["layer_policy"]["invoked_after_mean"] <= d["stack"]["off"]["invoked_after_mean"]


def test_bench_router_options():
    print("bench.py --config tiny --router sigmoid --groups 4,2", flush=True)
    d = _run("--config", "tiny", "--tokens", "16", "--steps", "3", "--warmup", "1", "--sweep-iters", "2", "--router", "sigmoid",
             "--groups", "4,2")
    assert "sigmoid-gated router" in d["config"]["workload"] and "group-limited router (2 of 4 groups)" in d["config"]["workload"]
    assert d["value"] > 0 and "cpu_baseline" not in d and "fp8_weights" not in d
    assert d["experts_invoked"]["after"] <= d["experts_invoked"]["before"]
