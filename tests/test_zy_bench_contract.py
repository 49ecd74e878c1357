"""The benchmark's command-line contract: one JSON line with the agreed fields on a GPU, a clear
refusal for more than one GPU and without a GPU (there is no CPU fallback)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          capture_output=True, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2", timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert not r.stdout.strip()


@pytest.mark.gpu
def test_json_line_has_the_agreed_fields():
    r = _bench("--steps", "40", "--warmup", "3")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "verified tok/s/GPU per spec step" and d["unit"] == "tok/s"
    assert d["n_gpus"] == 1 and d["steps"] == 40 and d["warmup"] == 3
    assert d["higher_is_better"] is True and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert d["vs_baseline"] is None and "workload" in d["config"]
    # value = B (K+1) tokens per step over the measured step time
    assert abs(d["value"] - 5 / d["ms_per_step"] * 1e3) / d["value"] < 1e-3
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    # achieved = algorithmic bytes per launch / mean launch duration of the dominant kernel
    assert abs(rf["achieved"] - rf["algorithmic_bytes_per_launch"] / (rf["avg_launch_us"] * 1e3)) / rf["achieved"] < 1e-3
    assert rf["traffic"] is None or rf["traffic"] > 0.8 * rf["algorithmic_bytes_per_launch"]
    # the launches timed by event pairs account for the step (one persistent kernel per step here)
    assert 0.5 < d["kernel_ms_per_step"] / d["ms_per_step"] <= 1.02   # (a slow host only lowers it)
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == "tok/s" and cb["cores"] >= 1 and cb["value"] > 0
    assert "steps" in cb["sample"]
    hist = d["accept_length_histogram"]
    assert sum(hist["counts"].values()) == hist["steps"]
    # the fixed-context points do not depend on --steps; the plain step and the other
    # configurations' fixed points ride on the same line
    assert [f["context"] for f in d["fixed_context"]] == [257, 2048, 4353]
    assert d["plain_step"]["ms_per_step"] > 0 and d["plain_step"]["spec_step_cost_ratio"] > 0.5
    assert rf["traffic_source"]
    sr = d["sampling_rules"]
    assert len(sr["cost_over_greedy"]) == 4 and all(0.9 < v < 1.5 for v in sr["cost_over_greedy"].values())
    sw = d["sweep"]
    assert [p["workload"].split(" context")[0] for p in sw] == ["c2 batch 16 K=6", "c4 batch 32 K=4", "c4 batch 128 K=8"]
    for p in sw:
        assert p["ms_per_step"] > 0 and 0 < p["hbm_frac"] < 1 and p["dominant_kernel"] in p["kernels"]
        assert 0 < p["projections"]["frac_of_mfma_bf16_peak"] < 1
