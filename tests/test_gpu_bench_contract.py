"""bench.py prints exactly one JSON line on stdout with the fields the measurement contract names
(run on the smallest workload, as a child process)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    return json.loads(lines[0]), r.stderr


def check_common(d, steps, warmup):
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == steps and d["warmup"] == warmup
    assert d["vs_baseline"] is None and d["dtype"] == "f32" and d["data"] == "synthetic"
    assert isinstance(d["config"]["workload"], str) and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in c, key
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0


def test_epoch_line_on_config_1():
    d, err = run_bench("--config", "1", "--steps", "5", "--warmup", "2")
    check_common(d, 5, 2)
    assert d["unit"] == "ms" and d["higher_is_better"] is False
    assert d["config"]["workload"].startswith("config 1")
    assert set(d["extra"]["phase_ms_per_epoch"]) == {"spmm", "gemm", "loss_elementwise_update"}
    assert "[bench" in err                                   # stage progress goes to stderr only


def test_spmm_line_on_a_small_graph():
    d, _ = run_bench("--config", "1", "--spmm", "--f", "16", "--steps", "5", "--warmup", "2")
    check_common(d, 5, 2)
    assert d["unit"] == "GB/s" and d["higher_is_better"] is True
    assert d["extra"]["nnz_matches_oracle"] is True
    assert d["extra"]["max_abs_err_vs_oracle"] <= 1e-4 * max(d["extra"]["rms_of_oracle"], 1e-30) * 10
