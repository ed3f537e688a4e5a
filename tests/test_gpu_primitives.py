"""The integer building blocks of graph construction (stable radix sort, exclusive prefix sum, removal of
equal neighbours) through the C-ABI, bit for bit against numpy's stable sort, cumsum and unique.  Sizes
straddle the kernels' tiles (2048 elements for the scan and the selection, 8192 keys for the sort)."""
import ctypes as C
import functools

import numpy as np
import pytest

from util import dev, host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@functools.lru_cache(maxsize=None)
def G():
    import paper_2005_03300_amd as g
    g.lib()
    return g


def keys_u64(kind, n, rs):
    if kind == "uniform":
        return rs.integers(0, 1 << 64, n, dtype=np.uint64)
    if kind == "few":                      # long runs of equal keys: stability is visible in the payload
        return rs.integers(0, 7, n, dtype=np.uint64) * np.uint64(0x0101010101010101)
    if kind == "edge":                     # row<<32|col keys of a small graph: four byte positions are constant
        return (rs.integers(0, 3000, n, dtype=np.uint64) << np.uint64(32)) | rs.integers(0, 3000, n, dtype=np.uint64)
    if kind == "sorted":
        return np.sort(rs.integers(0, 1 << 40, n, dtype=np.uint64))
    if kind == "reversed":
        return np.sort(rs.integers(0, 1 << 40, n, dtype=np.uint64))[::-1].copy()
    if kind == "equal":
        return np.full(n, 0xDEADBEEF12345678, dtype=np.uint64)
    raise ValueError(kind)


SORT_SIZES = [1, 2, 255, 256, 257, 8191, 8192, 8193, 100_003, 1_000_003]


@pytest.mark.parametrize("kind", ["uniform", "few", "edge", "sorted", "reversed", "equal"])
def test_radix_sort_keys_u64(kind):
    g = G()
    rs = np.random.default_rng(11)
    for n in SORT_SIZES:
        k = keys_u64(kind, n, rs)
        out, _ = g.gcn_radix_sort(dev(k.view(np.int64)))
        assert np.array_equal(host(out).view(np.uint64), np.sort(k, kind="stable")), (kind, n)


@pytest.mark.parametrize("width", [1, 2, 3])
@pytest.mark.parametrize("kind", ["uniform", "few", "edge"])
def test_radix_sort_pairs_u64_is_stable(kind, width):
    g = G()
    rs = np.random.default_rng(12 + width)
    for n in [1, 257, 8193, 300_007]:
        k = keys_u64(kind, n, rs)
        pay = rs.integers(-(1 << 31), 1 << 31, (n, width), dtype=np.int64).astype(np.int32)
        pay[:, 0] = np.arange(n, dtype=np.int32)            # input position: pins the order of equal keys
        order = np.argsort(k, kind="stable")
        out, pout = g.gcn_radix_sort(dev(k.view(np.int64)), dev(pay))
        assert np.array_equal(host(out).view(np.uint64), k[order]), (kind, width, n)
        assert np.array_equal(host(pout), pay[order]), (kind, width, n)


@pytest.mark.parametrize("end_bit", [1, 7, 8, 13, 32, 45, 63])
def test_radix_sort_ignores_bits_from_end_bit_up(end_bit):
    g = G()
    rs = np.random.default_rng(13)
    n = 50_001
    k = rs.integers(0, 1 << 64, n, dtype=np.uint64)
    pay = np.arange(n, dtype=np.int32)[:, None]
    mask = np.uint64((1 << end_bit) - 1)
    order = np.argsort(k & mask, kind="stable")             # bits above end_bit must not influence the order
    out, pout = g.gcn_radix_sort(dev(k.view(np.int64)), dev(pay), end_bit=end_bit)
    assert np.array_equal(host(pout)[:, 0], order.astype(np.int32))
    assert np.array_equal(host(out).view(np.uint64), k[order])


@pytest.mark.parametrize("end_bit", [32, 20, 9])
def test_radix_sort_u32_descending_keeps_input_order_of_ties(end_bit):
    g = G()
    rs = np.random.default_rng(14)
    for n in [1, 300, 8192, 70_001]:
        k = rs.integers(0, 50 if n > 300 else 5, n, dtype=np.uint32) * np.uint32(977)     # many ties
        if end_bit < 32:
            k |= rs.integers(0, 1 << (32 - end_bit), n, dtype=np.uint32) << np.uint32(end_bit)   # junk above end_bit
        pay = np.arange(n, dtype=np.int32)[:, None]
        low = (k & np.uint32((1 << end_bit) - 1 if end_bit < 32 else 0xFFFFFFFF)).astype(np.int64)
        order = np.argsort(-low, kind="stable")
        out, pout = g.gcn_radix_sort(dev(k.view(np.int32)), dev(pay), end_bit=end_bit, descending=True)
        assert np.array_equal(host(pout)[:, 0], order.astype(np.int32)), (end_bit, n)
        assert np.array_equal(host(out).view(np.uint32), k[order]), (end_bit, n)


def test_radix_sort_leaves_its_inputs_alone_and_rejects_bad_sizes():
    g = G()
    rs = np.random.default_rng(15)
    k = rs.integers(0, 1 << 64, 20_000, dtype=np.uint64)
    pay = rs.integers(0, 1 << 31, (20_000, 2), dtype=np.int64).astype(np.int32)
    kd, pd = dev(k.view(np.int64)), dev(pay)
    g.gcn_radix_sort(kd, pd)
    assert np.array_equal(host(kd).view(np.uint64), k) and np.array_equal(host(pd), pay)
    L = g.lib()
    s = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    o = torch.empty_like(kd)
    a, b = C.c_void_p(kd.data_ptr()), C.c_void_p(o.data_ptr())
    assert L.gcn_radix_sort(C.c_int64(10), 2, a, b, 0, None, None, 16, 0, s) == -1          # key size
    assert L.gcn_radix_sort(C.c_int64(10), 8, a, b, 5, a, b, 64, 0, s) == -1                 # payload size
    assert L.gcn_radix_sort(C.c_int64(10), 8, a, a, 0, None, None, 64, 0, s) == -1           # in place
    assert L.gcn_radix_sort(C.c_int64(-1), 8, a, b, 0, None, None, 64, 0, s) == -1
    assert L.gcn_radix_sort(C.c_int64(0), 8, None, None, 0, None, None, 64, 0, s) == 0       # nothing to do


@pytest.mark.parametrize("n", [1, 2, 2047, 2048, 2049, 4096, 100_000, 5_000_011])
def test_exclusive_scan_matches_cumsum(n):
    g = G()
    rs = np.random.default_rng(16)
    x = rs.integers(-(1 << 40), 1 << 40, n, dtype=np.int64)
    want = np.concatenate([np.zeros(1, np.int64), np.cumsum(x)[:-1]])
    xd = dev(x)
    assert np.array_equal(host(g.gcn_exclusive_scan_i64(xd)), want)
    assert np.array_equal(host(xd), x)
    g.gcn_exclusive_scan_i64(xd, out=xd)                     # in place
    assert np.array_equal(host(xd), want)


def test_exclusive_scan_wraps_like_two_s_complement():
    g = G()
    x = np.array([np.iinfo(np.int64).max, 1, 5, np.iinfo(np.int64).min, -7], dtype=np.int64)
    with np.errstate(over="ignore"):
        want = np.concatenate([np.zeros(1, np.uint64), np.cumsum(x.view(np.uint64))[:-1]]).view(np.int64)
    assert np.array_equal(host(g.gcn_exclusive_scan_i64(dev(x))), want)


@pytest.mark.parametrize("n", [1, 2, 2048, 2049, 77_777, 3_000_001])
@pytest.mark.parametrize("distinct", [1, 3, 1000, 1 << 62])
def test_unique_of_sorted_keys(n, distinct):
    g = G()
    rs = np.random.default_rng(17)
    k = np.sort(rs.integers(0, distinct, n, dtype=np.uint64))
    got = host(g.gcn_unique_u64(dev(k.view(np.int64)))).view(np.uint64)
    assert np.array_equal(got, np.unique(k)), (n, distinct)


def test_unique_keeps_first_of_each_run_of_unsorted_input():
    g = G()
    k = np.array([5, 5, 2, 2, 2, 5, 9, 9, 0], dtype=np.uint64)
    got = host(g.gcn_unique_u64(dev(k.view(np.int64)))).view(np.uint64)
    assert got.tolist() == [5, 2, 5, 9, 0]
    assert g.gcn_unique_u64(torch.empty(0, dtype=torch.int64, device="cuda")).numel() == 0
