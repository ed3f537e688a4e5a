"""The five named workloads and scaled-down versions of them.

Configs 3, 4 and 5 are synthetic stand-ins with the vertex count, edge count, feature width
and label count of the paper's Reddit, Amazon and Protein datasets (table "Datasets used in
our experiments"); configs 1 and 2 are an Erdos-Renyi toy and an R-MAT scale-20 matrix.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

from . import dense, graphs


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    kind: str                 # "er" | "rmat" | "chunglu"
    n: int
    m_raw: int                # endpoint pairs drawn (before any cleaning)
    dims: tuple               # f^0 .. f^{L_w}; for the SpMM-only config just (f,)
    n_classes: int
    features: str             # "uniform" | "normal"
    rmat_scale: int = 0
    gamma: float = 0.0
    max_degree: float = 0.0
    permute: bool = True


CONFIGS = {
    1: Workload("er4096_gcn_64_16_8", "er", 4096, 4096 * 16 // 2, (64, 16, 8), 8, "uniform",
                permute=False),
    2: Workload("rmat20_spmm_f128", "rmat", 1 << 20, 16 << 20, (128,), 0, "uniform", rmat_scale=20),
    # m_raw of 3-5 is chosen so that, after duplicate removal, the number of distinct
    # unordered pairs lands near the dataset's edge count / 2.
    3: Workload("chunglu_reddit_gcn_602_16_16_41", "chunglu", 232_965, 59_450_000,
                (602, 16, 16, 41), 41, "normal", gamma=2.1, max_degree=20_000.0),
    4: Workload("rmat_amazon_gcn_300_16_16_24", "rmat", 14_249_639, 121_500_000,
                (300, 16, 16, 24), 24, "normal", rmat_scale=24),
    5: Workload("chunglu_protein_gcn_128_16_16_256", "chunglu", 8_745_542, 656_500_000,
                (128, 16, 16, 256), 256, "normal", gamma=2.3, max_degree=50_000.0),
}


def scaled(cfg: int | Workload, shrink: int) -> Workload:
    """The same recipe with ``n`` and the number of drawn pairs divided by ``shrink`` (a power
    of two for R-MAT), so mean degree and skew are kept while the oracle stays fast."""
    w = CONFIGS[cfg] if isinstance(cfg, int) else cfg
    if shrink <= 1:
        return w
    bits = int(round(math.log2(shrink)))
    n = max(8, w.n // shrink)
    return dataclasses.replace(
        w, name=f"{w.name}_div{shrink}", n=n, m_raw=max(8, w.m_raw // shrink),
        rmat_scale=max(3, w.rmat_scale - bits) if w.kind == "rmat" else 0,
        max_degree=(max(min(w.max_degree, 0.5 * n), 2.5 * w.m_raw / w.n)
                    if w.kind == "chunglu" else 0.0))


def make_graph(w: Workload, seed: int = 0):
    """Return ``(n, src, dst)``: the raw directed endpoint pairs of workload ``w``."""
    if w.kind == "er":
        src, dst = graphs.erdos_renyi(w.n, w.m_raw, seed)
    elif w.kind == "rmat":
        n_keep = w.n if w.n < (1 << w.rmat_scale) else None
        src, dst = graphs.rmat(w.rmat_scale, w.m_raw, n_keep=n_keep, seed=seed)
    elif w.kind == "chunglu":
        src, dst = graphs.chung_lu(w.n, w.m_raw, w.gamma, w.max_degree, seed)
    else:
        raise ValueError(w.kind)
    if w.permute:
        src, dst = graphs.relabel(w.n, src, dst, seed)
    return w.n, np.ascontiguousarray(src), np.ascontiguousarray(dst)


def make_model_inputs(w: Workload, seed: int = 0, features: bool = True):
    """Return ``(H0, labels, weights)`` for workload ``w`` (``labels``/``weights`` are None for
    the SpMM-only workload)."""
    f0 = w.dims[0]
    H0 = None
    if features:
        H0 = (dense.uniform_features if w.features == "uniform" else dense.normal_features)(w.n, f0, seed)
    if len(w.dims) == 1:
        return H0, None, None
    return H0, dense.labels(w.n, w.n_classes, seed), dense.glorot_weights(w.dims, seed)
