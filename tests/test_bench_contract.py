"""bench.py's contract with the driver: one JSON line with the agreed keys on one GPU, a refusal for more."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    for extra, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *extra], capture_output=True, text=True,
                           env={**os.environ, **env})
        assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def _check_record(j, name, bound):
    for k in ("value", "unit", "ms_per_step", "dtype", "config", "roofline", "cpu_baseline"):
        assert k in j, (name, k)
    assert j["config"]["workload"] == name and "model" not in j["config"] and j["dtype"] == "bf16"
    assert abs(j["value"] - j["config"]["B"] / (j["ms_per_step"] * 1e-3)) < 1e-6 * j["value"]
    ro = j["roofline"]
    assert ro["bound"] == bound and ro["unit"] == ("GB/s" if bound == "hbm" else "TFLOP/s")
    assert ro["peak"] == (8000.0 if bound == "hbm" else 2500.0)
    assert abs(ro["frac"] - ro["achieved"] / ro["peak"]) < 1e-12 and 0.2 < ro["frac"] < 1.0
    # the whole step (LM head + tail + launch gaps) cannot beat its dominant kernel; the two are timed in separate
    # passes of a few steps each, hence the margin
    assert 0.0 < ro["step_frac"] <= ro["frac"] * 1.10 and ro["kernel_ms"] <= j["ms_per_step"] * 1.10
    if ro["traffic"] is not None:
        assert ro["traffic"] > 0.99 * ro["algorithmic_bytes"] and "traffic_source" in ro
    cb = j["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample_matches_gpu"] is True


@pytest.mark.gpu
def test_default_line_headlines_the_largest_workload_and_carries_the_others():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "5", "--warmup", "2"],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "workloads"):
        assert k in j, k
    assert j["n_gpus"] == 1 and j["steps"] == 5 and j["warmup"] == 2 and j["vs_baseline"] is None
    _check_record(j, "70b_b128_k64", "mfma")
    bounds = {"8b_b1_k16": "hbm", "70b_b8_k32": "hbm", "70b_b1_k32": "hbm", "70b_b1_k64": "hbm", "8b_b32_k32": "mfma"}
    assert set(j["workloads"]) == set(bounds)
    for name, bound in bounds.items():
        _check_record(j["workloads"][name], name, bound)
    assert j["workloads"]["8b_b1_k16"]["roofline"]["kernel"] == "lm_head_stream16_bf16"


@pytest.mark.gpu
def test_single_workload_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "8b_b1_k16", "--steps", "5",
                        "--warmup", "2"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    assert "workloads" not in j and j["steps"] == 5
    _check_record(j, "8b_b1_k16", "hbm")
