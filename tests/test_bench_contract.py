"""The benchmark's command-line contract: one JSON line with the agreed fields; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=timeout, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2", timeout=60)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "one GPU" in r.stderr


@pytest.mark.gpu
def test_default_line_has_the_contract_fields():
    r = _run("--steps", "20", "--warmup", "3")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 3 and d["unit"] == "TFLOP/s" and d["vs_baseline"] is None
    assert d["dtype"] == "bf16" and d["data"] == "synthetic" and "workload" in d["config"] and "model" not in d["config"]
    assert 100 < d["value"] < 2516.6                                   # below the dense bf16 MFMA peak
    # value = nominal work of the three ops / sum of the single-stream kernel medians; the wall time of the
    # single-stream step loop contains the same kernels plus the gaps between launches
    ks = d["kernel_sum"]["us"]
    assert abs(ks - sum(k["us"] * k["count"] for k in d["kernels"].values())) < 0.05
    assert abs(d["value"] - 3 * 14.797 / (ks * 1e-3)) / d["value"] < 0.01
    assert d["config"]["streams"] == 1 and d["batches"] >= 5 and len(d["step_wall"]["ms_per_step_batches"]) == d["batches"]
    assert ks * 1e-3 <= d["ms_per_step"] * 1.02 and d["step_wall"]["tflops"] <= d["value"] * 1.02
    assert d["three_stream_step"]["tflops"] > 0
    assert set(d["cfg1_us"]) >= {"fwd", "bwd_data", "bwd_filters"} and all(0 < d["cfg1_us"][k] < 1000 for k in ("fwd", "bwd_data", "bwd_filters"))
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "mfma" and roof["peak"] == 2516.6 and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    # measured HBM bytes (from the committed counter summary; null when there is none) are not below the algorithmic ones
    assert roof["traffic"] is None or roof["traffic"] >= 51_527_680
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["unit"] == "TFLOP/s" and 0 < cpu["value"] < 1
    assert cpu["cpu_model"] and cpu["one_thread"]["cores"] == 1 and 0 < cpu["one_thread"]["value"] <= cpu["value"] * 1.5
