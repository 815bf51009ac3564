"""The bench's command line (CPU side): more than one GPU is refused with a message, a machine without a GPU is
reported, and a GPU run (marked gpu) prints exactly one JSON line with the fields the contract names."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, timeout=600):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_contract_fields():
    r = _run("--steps", "20", "--warmup", "3", "--no-lm-head")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 3 and d["data"] == "synthetic"
    assert d["value"] > 0 and abs(d["value"] - d["config"]["committed_tokens_per_step"] / (d["ms_per_step"] * 1e-3)) < 1e-6 * d["value"]
    roof = d["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] >= 1
    assert "workload" in d["config"] and "model" not in d["config"]
    # the headline is the largest single-GPU workload, and all three calls of the step carry a roofline entry
    assert d["config"]["workload"].startswith("cfg5") and "layers=32" in d["config"]["workload"]
    assert roof["bound"] == "hbm" and "not measured in this run" in roof.get("traffic_source", "not measured in this run")
    kinds = [o["kernel"].split(" ")[0] for o in roof["others"]]
    assert kinds == ["sdllm_confidence_unmask", "sdllm_kv_append"]
    for o in roof["others"]:
        assert o["launch_ms"] > 0 and abs(o["frac"] - o["achieved"] / o["peak"]) < 1e-12
        assert abs(o["achieved"] - o["algorithmic_bytes"] / o["launch_ms"] / 1e6) < 1e-6 * o["achieved"]
    assert roof["others"][0]["alu_roof"]["roof_ms"] > 0
    ex = d["exclusions"]
    assert ex["gpu_matches_oracle_outside_band"] is True and ex["sequences_checked"] >= 1
