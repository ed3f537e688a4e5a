"""The seeded synthetic inputs: reproducible, independent of the thread count, and with the shapes and
skew that the design notes state for the stand-in workloads."""
import numpy as np
import pytest

import synth
from synth import graphs


def test_streams_are_reproducible_and_chunk_independent():
    a = synth.erdos_renyi(5000, 200_000, seed=3)
    b = synth.erdos_renyi(5000, 200_000, seed=3)
    c = synth.erdos_renyi(5000, 200_000, seed=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[0], c[0])
    x = synth.normal_features(1000, 7, 5)
    assert np.array_equal(x, synth.normal_features(1000, 7, 5))
    assert x.dtype == np.float32 and x.shape == (1000, 7)
    assert not np.array_equal(x, synth.normal_features(1000, 7, 6))


def test_feature_and_label_distributions():
    u = synth.uniform_features(200_000, 4, 1)
    assert u.min() >= -1.0 and u.max() < 1.0 and abs(float(u.mean())) < 0.01
    z = synth.normal_features(200_000, 4, 2)
    assert abs(float(z.mean())) < 0.01 and abs(float(z.std()) - 1.0) < 0.01
    y = synth.labels(100_000, 41, 3)
    assert y.dtype == np.int32 and y.min() == 0 and y.max() == 40
    counts = np.bincount(y, minlength=41)
    assert counts.min() > 0.8 * 100_000 / 41
    ws = synth.glorot_weights((602, 16, 41), 4)
    assert [w.shape for w in ws] == [(602, 16), (16, 41)]
    for w, (fi, fo) in zip(ws, ((602, 16), (16, 41))):
        bound = np.sqrt(6.0 / (fi + fo))
        assert np.abs(w).max() <= bound and np.abs(w).max() > 0.9 * bound


def test_rmat_quadrant_probabilities_and_skew():
    scale, m = 12, 400_000
    src, dst = graphs.rmat(scale, m, seed=1)
    assert src.min() >= 0 and src.max() < (1 << scale) and dst.max() < (1 << scale)
    top_s, top_d = src >> (scale - 1), dst >> (scale - 1)          # the first quadrant choice
    frac = [np.mean((top_s == i) & (top_d == j)) for i in (0, 1) for j in (0, 1)]   # a, b, c, d
    np.testing.assert_allclose(frac, [0.57, 0.19, 0.19, 0.05], atol=0.005)
    deg = np.bincount(src, minlength=1 << scale)
    assert deg.max() > 50 * deg.mean()                              # heavy hubs
    kept = graphs.rmat(scale, m, n_keep=3000, seed=1)
    assert kept[0].max() < 3000 and kept[1].max() < 3000 and len(kept[0]) < m


def test_chung_lu_degrees_follow_the_weights_and_the_cap():
    n, m, cap = 20_000, 1_000_000, 2_000.0
    w = graphs.chung_lu_weights(n, 2.1, m, cap)
    w = np.asarray(w, np.float64)
    expected = w / w.sum() * 2 * m
    assert abs(expected.max() - cap) < 0.02 * cap and np.all(np.diff(expected) <= 1e-9)   # capped, descending
    src, dst = graphs.chung_lu(n, m, 2.1, cap, seed=2)
    deg = np.bincount(src, minlength=n) + np.bincount(dst, minlength=n)
    top = slice(0, 50)
    assert abs(deg[top].sum() / expected[top].sum() - 1.0) < 0.05
    with pytest.raises(Exception):
        graphs.chung_lu_weights(n, 2.1, m, 10.0)                    # cap below the mean degree


def test_relabelling_is_a_permutation_and_scaled_configs_keep_mean_degree():
    src, dst = graphs.ring(1000)
    s2, d2 = graphs.relabel(1000, src, dst, seed=5)
    assert sorted(set(s2.tolist())) == list(range(1000))
    a = set(zip(src.tolist(), dst.tolist()))
    b = set(zip(s2.tolist(), d2.tolist()))
    assert len(b) == len(a) and a != b
    for cfg in (3, 4, 5):
        full, small = synth.CONFIGS[cfg], synth.scaled(cfg, 64)
        assert abs(small.m_raw / small.n - full.m_raw / full.n) < 0.02 * full.m_raw / full.n
    assert synth.scaled(2, 1) is synth.CONFIGS[2]


def test_named_workloads_have_the_stated_shapes():
    c = synth.CONFIGS
    assert (c[1].n, c[1].dims) == (4096, (64, 16, 8))
    assert (c[2].n, c[2].m_raw, c[2].dims) == (1 << 20, 16 << 20, (128,))
    assert (c[3].n, c[3].dims, c[3].n_classes) == (232_965, (602, 16, 16, 41), 41)
    assert (c[4].n, c[4].dims, c[4].n_classes) == (14_249_639, (300, 16, 16, 24), 24)
    assert (c[5].n, c[5].dims, c[5].n_classes) == (8_745_542, (128, 16, 16, 256), 256)
