"""The benchmark's command-line contract: one JSON line with the agreed keys; more than one GPU is
refused with a message (this build is one EP rank's share on one GPU)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_keys():
    r = run_bench("--workload", "C1", "--steps", "3", "--warmup", "1", "--cpu-tokens", "256")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["unit"] == "TFLOP/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("C1") and "model" not in d["config"]
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["integer_outputs_match"] is True
    assert d["value"] > 0 and d["ms_per_step"] > 0
    assert cpu["parity"] is True and cpu["rows_above_row_bar"] == 0 and cpu["worst_element_over_storage_format_bound"] <= 1.0
    assert cpu["host_cpus"] >= cpu["cores"] >= 1
    # one roofline object per kernel of the step, each recomputable from its own fields
    assert set(d["rooflines"]) == {"down", "combine", "permute_with_gather", "row_gather_alone", "route"}
    for key, r in list(d["rooflines"].items()) + [("gate_up", roof)]:
        assert r["bound"] in ("mfma", "hbm", "alu") and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9, key
        assert r["avg_launch_ms"] > 0
    assert roof["per_launch"][0]["nonempty_groups"] == d["config"]["nonempty_groups"] == 8
    assert abs(roof["flops_per_launch"] / (roof["avg_launch_ms"] * 1e-3) / 1e12 - roof["achieved"]) < 1e-6 * roof["achieved"]
    # the other four workloads are timed in the default run as well
    assert set(d["other_workloads"]) == {"C2", "C3", "C4", "C5"}
    c3 = d["other_workloads"]["C3"]
    assert c3["gate_up"]["frac"] > 0 and c3["down"]["frac"] > 0 and c3["R"] > 8192
    assert d["ffn_training_step"]["ms"]["backward"] > 0
