"""The entry point that allocates nothing (gcn_spmm_static) against the existing one (gcn_spmm), through the C ABI:
two calls in a row on the fixed scratch array, the second with a smaller input, both bit-identical to gcn_spmm
over the same schedule and within the parity bar of the automatically chosen one and of the oracle."""
import numpy as np
import pytest

import oracle
import synth
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _lib():
    import paper_2005_03300_amd as g
    g.lib()
    return g


def _pair(g, name_cfg, shrink, f, trans, seed, epilogue=0):
    """One product through both entry points on the graph of config `name_cfg` shrunk `shrink` times."""
    n, src, dst = synth.make_graph(synth.scaled(name_cfg, shrink))
    fl = g.SYMMETRISE | g.ADD_SELF_LOOPS | g.NORM_SYM | g.BUILD_TRANSPOSE
    a = g.gcn_csr_create(n, dev(src), dev(dst), fl)
    X = synth.normal_features(n, f, seed)
    Xd = dev(X)
    Zprev = dev(synth.normal_features(n, f, seed + 1)) if epilogue == g.EPI_MASK else None
    Zs = torch.full((n, f), float("nan"), device="cuda")
    g.gcn_spmm_static(a, trans, Xd, Zs, epilogue, Zprev)
    torch.cuda.synchronize()
    # the existing entry point, automatic schedule: the parity bar
    Za = torch.empty(n, f, device="cuda")
    g.gcn_spmm(a, trans, Xd, Za, epilogue, Zprev)
    assert_close(host(Zs), host(Za), f"static vs gcn_spmm (automatic schedule), f={f}")
    # the existing entry point forced to the same schedule: bit for bit
    g.gcn_config(g.CFG_SPMM_ALGO, 2)
    g.gcn_config(g.CFG_SPMM_BLOCKS, 1)
    g.gcn_config(g.CFG_PATTERN_SPMM, 0)           # the stored values, as the static entry point reads them
    try:
        Zf = torch.empty(n, f, device="cuda")
        g.gcn_spmm(a, trans, Xd, Zf, epilogue, Zprev)
    finally:
        g.gcn_config(g.CFG_SPMM_ALGO, 0)
        g.gcn_config(g.CFG_SPMM_BLOCKS, 0)
        g.gcn_config(g.CFG_PATTERN_SPMM, 2)
    assert torch.equal(Zs, Zf), f"static differs from the same schedule of gcn_spmm, f={f}"
    if epilogue == 0:
        A = oracle.build_csr(n, src, dst)
        assert_close(host(Zs), oracle.spmm(A, X), f"static vs oracle, f={f}")
    a.close()


def test_static_spmm_two_calls_in_a_row_second_smaller():
    g = _lib()
    _pair(g, 3, 32, 64, 0, 11)                    # 3.6 M entries, heavy rows crossing many wavefronts, f = 64
    _pair(g, 2, 64, 16, 1, 12)                    # smaller graph, narrower operand, transposed arrays; the array
    _pair(g, 1, 1, 8, 0, 13, epilogue=2)          # still holds what the call before left there; then tiny + mask


def test_static_spmm_rejects_what_does_not_fit():
    g = _lib()
    n, src, dst = synth.make_graph(synth.scaled(3, 32))
    a = g.gcn_csr_create(n, dev(src), dev(dst), g.SYMMETRISE | g.ADD_SELF_LOOPS | g.NORM_SYM)
    f = 16 * (1 + (16 << 20) // (4 * 16 * ((a.nnz + 511) // 512)))          # first multiple of 16 that no longer fits
    X = torch.zeros(n, f, device="cuda")
    Z = torch.empty(n, f, device="cuda")
    with pytest.raises(g.GcnError) as e:
        g.gcn_spmm_static(a, 0, X, Z)
    assert e.value.code == -5 and "gcn_spmm" in str(e.value)
    with pytest.raises(g.GcnError) as e:                                   # built without the transpose
        g.gcn_spmm_static(a, 1, X[:, :16].contiguous(), Z[:, :16].contiguous())
    assert e.value.code == -3
    a.close()
