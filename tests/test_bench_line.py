"""The benchmark's own contract: one JSON line with the fields the measurement record is read from, and a
refusal of more than one GPU.  The GPU case runs a two-layer version of the headline workload in a child
process (a second or two of GPU time)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.gpu
def test_bench_line_fields():
    r = run_bench("--layers", "2", "--steps", "2", "--warmup", "1", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "roofline_other", "peaks_measured"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 2 and j["warmup"] == 1 and j["dtype"] == "bf16" and j["data"] == "synthetic"
    assert j["config"]["workload"] == "cfg2_mistral7b" and j["config"]["layers"] == 2 and "model" not in j["config"]
    assert j["value"] > 0 and j["ms_per_step"] > 0
    # tokens per second of the whole job: batch * doc_len / step time
    assert abs(j["value"] - j["config"]["batch"] * j["config"]["doc_len"] / (j["ms_per_step"] * 1e-3)) <= 1e-3 * j["value"]
    ro = j["roofline"]
    for key in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "avg_launch_ms"):
        assert key in ro, key
    assert ro["bound"] == "mfma" and ro["unit"] == "TFLOP/s" and ro["peak"] == 2500.0
    assert abs(ro["frac"] - ro["achieved"] / ro["peak"]) < 1e-3
    assert abs(ro["achieved"] - ro["algorithmic_flops_per_launch"] / (ro["avg_launch_ms"] * 1e-3) / 1e12) <= 1e-2 * ro["achieved"]
    steps = {o["step"]: o for o in j["roofline_other"]}
    assert set(steps) == {"a2", "a3", "a4"}
    for s in ("a2", "a4"):
        o = steps[s]
        assert o["bound"] in ("hbm", "mfma") and o["avg_launch_ms"] > 0
        assert abs(o["frac"] - o["achieved"] / o["peak"]) < 1e-3
    a4 = steps["a4"]
    assert abs(a4["achieved"] - a4["algorithmic_bytes_per_launch"] / (a4["avg_launch_ms"] * 1e-3) / 1e9) <= 1e-2 * a4["achieved"]
    pk = j["peaks_measured"]
    assert 1000.0 < pk["copy_GBs"] < 8000.0 and 500.0 < pk["mfma_only_bf16_TFLOPs"] < 2500.0
    # every fraction is also given against what the same run measured as reachable
    assert abs(ro["frac_of_measured_peak"] - ro["achieved"] / pk["mfma_only_bf16_TFLOPs"]) < 1e-3
    assert abs(a4["frac_of_measured_peak"] - a4["achieved"] / pk["copy_GBs"]) < 1e-3
    a2 = steps["a2"]
    reached = pk["mfma_only_bf16_TFLOPs"] if a2["unit"] == "TFLOP/s" else pk["copy_GBs"]
    assert abs(a2["frac_of_measured_peak"] - a2["achieved"] / reached) < 1e-3
