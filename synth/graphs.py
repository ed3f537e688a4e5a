"""Raw edge lists (int32 ``src``, ``dst``), possibly with duplicates and self-loops.

Cleaning the list (symmetrising, removing duplicates, inserting the diagonal) is part of the
method and is done by the consumers, never here.
"""
from __future__ import annotations

import numpy as np

from .rng import STREAM_EDGES, STREAM_PERM, for_chunks, stream_rng


def _concat(parts):
    src = np.concatenate([p[0] for p in parts]) if parts else np.zeros(0, np.int32)
    dst = np.concatenate([p[1] for p in parts]) if parts else np.zeros(0, np.int32)
    return np.ascontiguousarray(src, np.int32), np.ascontiguousarray(dst, np.int32)


def erdos_renyi(n: int, m: int, seed: int = 0):
    """``m`` endpoint pairs drawn uniformly and independently from ``[0,n)^2``."""
    def draw(c, s, e):
        g = stream_rng(seed, STREAM_EDGES, c)
        k = e - s
        return (g.integers(0, n, size=k, dtype=np.int64).astype(np.int32),
                g.integers(0, n, size=k, dtype=np.int64).astype(np.int32))
    return _concat(for_chunks(m, draw))


def rmat(scale: int, m: int, a=0.57, b=0.19, c=0.19, d=0.05, n_keep: int | None = None, seed: int = 0):
    """R-MAT: each of ``m`` edges picks one quadrant per bit level with probabilities
    (a, b, c, d); quadrants c and d set the source bit, b and d the destination bit.
    Edges with an endpoint ``>= n_keep`` are discarded when ``n_keep`` is given."""
    assert abs(a + b + c + d - 1.0) < 1e-9

    def draw(ci, s, e):
        g = stream_rng(seed, STREAM_EDGES, ci)
        k = e - s
        u = np.zeros(k, np.int64)
        v = np.zeros(k, np.int64)
        for _ in range(scale):
            r = g.random(k)
            ubit = r >= (a + b)
            vbit = ((r >= a) & (r < a + b)) | (r >= a + b + c)
            u = (u << 1) | ubit
            v = (v << 1) | vbit
        if n_keep is not None:
            keep = (u < n_keep) & (v < n_keep)
            u, v = u[keep], v[keep]
        return u.astype(np.int32), v.astype(np.int32)
    return _concat(for_chunks(m, draw))


def directed_rmat(scale: int, m: int, seed: int = 0):
    """Same generator; the name marks call sites whose consumers must NOT symmetrise."""
    return rmat(scale, m, seed=seed)


def chung_lu_weights(n: int, gamma: float, m_pairs: int, max_expected_degree: float):
    """Power-law vertex weights ``w_i = (i + i0)^(-1/(gamma-1))``; the offset ``i0`` is the
    smallest one for which the heaviest vertex's expected degree ``2 m w_0 / sum(w)`` stays
    at or below ``max_expected_degree``."""
    alpha = 1.0 / (gamma - 1.0)
    idx = np.arange(n, dtype=np.float64)
    if 2.0 * m_pairs / n >= max_expected_degree:
        raise ValueError("max_expected_degree must exceed the mean degree 2 m / n")

    def top_degree(i0):
        w = (idx + i0) ** (-alpha)
        return 2.0 * m_pairs * w[0] / w.sum()

    lo, hi = 1e-9, 1.0
    while top_degree(hi) > max_expected_degree:
        hi *= 2.0
    if top_degree(lo) <= max_expected_degree:
        hi = lo
    else:
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            if top_degree(mid) > max_expected_degree:
                lo = mid
            else:
                hi = mid
    return (idx + hi) ** (-alpha)


def chung_lu(n: int, m_pairs: int, gamma: float, max_expected_degree: float, seed: int = 0):
    """``m_pairs`` endpoint pairs, both endpoints drawn independently with probability
    proportional to the power-law weights (inverse-CDF sampling)."""
    w = chung_lu_weights(n, gamma, m_pairs, max_expected_degree)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]

    def draw(c, s, e):
        g = stream_rng(seed, STREAM_EDGES, c)
        k = e - s
        u = np.searchsorted(cdf, g.random(k), side="right")
        v = np.searchsorted(cdf, g.random(k), side="right")
        np.minimum(u, n - 1, out=u)
        np.minimum(v, n - 1, out=v)
        return u.astype(np.int32), v.astype(np.int32)
    return _concat(for_chunks(m_pairs, draw))


def relabel(n: int, src: np.ndarray, dst: np.ndarray, seed: int = 0):
    """Seeded random renaming of the vertices (the paper permutes vertices before training,
    section "Datasets and Compute Platform")."""
    perm = stream_rng(seed, STREAM_PERM).permutation(n).astype(np.int32)
    return perm[src], perm[dst]


def star(n: int):
    """Vertex 0 joined to every other vertex: one row with n nonzeros after cleaning."""
    dst = np.arange(1, n, dtype=np.int32)
    return np.zeros(n - 1, np.int32), dst


def ring(n: int):
    src = np.arange(n, dtype=np.int32)
    return src, ((src + 1) % n).astype(np.int32)
