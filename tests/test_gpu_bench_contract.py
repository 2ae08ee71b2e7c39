"""bench.py's line, on a reduced row count so that it takes seconds: the keys the measurement contract names are
there in every mode, the values are consistent with each other, and the modes beside the default one still run."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*flags):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *flags], capture_output=True, text=True, cwd=ROOT,
                       timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


def _check_contract(d, steps, warmup):
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == steps and d["warmup"] == warmup
    assert d["data"] == "synthetic" and d["vs_baseline"] is None
    assert isinstance(d["config"]["workload"], str) and "model" not in d["config"]
    rf = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in rf, key
    assert rf["bound"] in ("hbm", "mfma", "alu")
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) <= 1e-3
    assert d["ms_per_step"] > 0 and d["value"] > 0


def test_planted_workload_line_with_cpu_baseline():
    d = _bench("--config", "2", "--n", "65536", "--steps", "2", "--warmup", "1", "--cpu-sample-rows", "16384")
    _check_contract(d, 2, 1)
    assert d["unit"] == "GB/s" and d["higher_is_better"] is True and d["roofline"]["bound"] == "hbm"
    # value is the step's algorithmic bytes over its time
    assert abs(d["value"] - d["config"]["algorithmic_GB_per_step"] / (d["ms_per_step"] * 1e-3)) <= 0.02 * d["value"]
    cb = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cb, key
    assert cb["kind"] == "oracle" and cb["cores"] >= 1
    same = cb["same_inputs"]
    assert same["gpu_ms"] > 0 and same["oracle_seconds"] > 0 and same["max_rel_diff_ritz_values"] <= 1e-4
    for name in ("hvp_project", "hvp_expand", "reorth_dot", "reorth_sub", "ritz_vectors", "step", "step_project",
                 "step_complement", "step_apply"):
        assert d["phases"][name]["launches"] >= 1


def test_outer_iteration_mode():
    d = _bench("--config", "2", "--n", "65536", "--outer", "--steps", "2", "--warmup", "1", "--no-cpu-baseline")
    _check_contract(d, 2, 1)
    assert "outer iteration" in d["config"]["workload"]
    assert d["phases"]["step"]["launches"] == 10 and d["phases"]["admm"]["launches"] == 2


def test_softmax_ggn_line():
    d = _bench("--config", "3", "--steps", "2", "--warmup", "1", "--no-cpu-baseline")
    _check_contract(d, 2, 1)
    assert d["roofline"]["bound"] == "mfma" and d["roofline"]["unit"] == "TFLOP/s" and d["higher_is_better"] is False


def test_traffic_model_mode():
    d = _bench("--config", "2", "--n", "65536", "--traffic-model")
    assert set(d["kernels_of_one_step"]) == {"ritz_vectors", "step_project", "step_complement", "step_apply"}
    for v in d["traffic_model"].values():
        assert v["avg_ms"] > 0 and v["GBps"] > 0
