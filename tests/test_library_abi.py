"""The C-ABI library loads without a GPU and exports every function include/gcn.h declares.
No compute entry point is called here."""
import os

import pytest

import paper_2005_03300_amd as g


def test_library_is_built_in_tree():
    assert os.path.exists(g.library_path()), "run `python -m paper_2005_03300_amd.build` first"


def test_every_declared_symbol_is_exported():
    L = g.lib()
    names = g.exported_symbols()
    assert len(names) >= 20 and "gcn_spmm" in names and "gcn_epoch" in names
    for name in names:
        assert hasattr(L, name), f"{name} is declared in gcn.h but not exported"


def test_host_only_calls():
    assert "gfx950" in g.gcn_version()
    with pytest.raises(g.GcnError) as e:
        g.gcn_config(12345, 1)
    assert e.value.code == -1 and "unknown config key" in str(e.value)
    g.gcn_config(g.CFG_SPMM_ALGO, 2)
    g.gcn_config(g.CFG_SPMM_ALGO, 0)
    # workspace sizing is pure host arithmetic: sum over layers of H (last layer: Z), T, G plus the shared S,
    # the scaled-operand buffer of the same size and the region for partial sums
    n, dims = 1000, [64, 16, 8]
    want = 0
    r = lambda e: (e * 4 + 255) // 256 * 256
    for l in range(2):
        fo = dims[l + 1]
        want += r(n * fo) + r(n * fo) + r(n * fo)          # H (or last Z), T, G
    want += 2 * r(n * 16)
    want += 2048 * 8            # partial sums of the reductions over n: here the loss's 2048 doubles are the largest
    assert g.gcn_epoch_workspace_bytes(n, dims, g.ORDER_GEMM_FIRST) == want
    assert g.gcn_epoch_workspace_bytes(n, [64, 0, 8], 0) == 0


def test_binding_does_not_touch_the_oracle():
    import sys
    here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for fn in ("__init__.py", "binding.py", "build.py"):
        text = open(os.path.join(here, "paper_2005_03300_amd", fn)).read()
        assert "import oracle" not in text and "from oracle" not in text
    for fn in os.listdir(os.path.join(here, "oracle")):
        if fn.endswith((".py", ".c")):
            text = open(os.path.join(here, "oracle", fn)).read()
            assert "paper_2005_03300_amd" not in text and "gcn.h" not in text


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""
