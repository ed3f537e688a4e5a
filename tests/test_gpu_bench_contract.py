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
    d, err = run_bench("--config", "1", "--epoch", "--steps", "5", "--warmup", "2")
    check_common(d, 5, 2)
    assert d["unit"] == "ms" and d["higher_is_better"] is False
    assert d["config"]["workload"].startswith("config 1")
    assert set(d["extra"]["phase_ms_per_epoch"]) == {"spmm", "gemm", "loss_elementwise_update"}
    assert "[bench" in err                                   # stage progress goes to stderr only


def test_spmm_line_on_a_small_graph():
    d, _ = run_bench("--config", "1", "--f", "16", "--steps", "5", "--warmup", "2")
    check_common(d, 5, 2)
    assert d["unit"] == "GB/s" and d["higher_is_better"] is True
    assert d["config"]["workload"].startswith("config 1: stand-alone SpMM")
    assert d["extra"]["sampled_rows_match_full_product"] is True
    assert d["extra"]["max_abs_err_vs_oracle"] <= 1e-4 * max(d["extra"]["rms_of_oracle"], 1e-30)
    assert d["extra"]["event_brackets"] == 10 and d["roofline"]["traffic"] is None      # no counter profile for this graph


def test_default_workload_is_the_largest_config():
    """Without flags the benchmark times the stand-alone SpMM on config 5 (checked from the argument parser: the
    run itself takes minutes and is the driver's)."""
    import re
    text = open(os.path.join(ROOT, "bench.py")).read()
    assert re.search(r'"--config", type=int, default=5', text)
    assert "action=\"store_true\"" in text and '"--epoch"' in text


def test_stored_traffic_figures_name_the_schedule_they_were_measured_on():
    """roofline.traffic is a counter measurement stored in bench.py; each figure names the schedule (as the
    library describes it) it was taken on, and the library must still take that schedule for that workload --
    otherwise the figure is stale and has to be measured again.  Config 2 is checked here (two seconds); the
    config 3, 4 and 5 figures are checked in the full-size parity tests, which build those graphs anyway."""
    import numpy as np
    import torch
    sys.path.insert(0, ROOT)
    import bench
    import paper_2005_03300_amd as g
    import synth
    w = synth.CONFIGS[2]
    n, src, dst = synth.make_graph(w)
    a = g.gcn_csr_create(n, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(),
                         g.SYMMETRISE | g.ADD_SELF_LOOPS | g.NORM_SYM | g.BUILD_TRANSPOSE)
    meas = bench.MEASURED_TRAFFIC[(w.name, 128)]
    assert meas["schedule"] == g.gcn_spmm_describe(a, 0, 128), (meas["schedule"], g.gcn_spmm_describe(a, 0, 128))
    assert os.path.exists(os.path.join(ROOT, meas["profile"]))
    a.close()
