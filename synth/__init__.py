"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only *draws* inputs (edge lists, feature matrices, labels, initial
weights).  It contains none of the method's arithmetic: no CSR construction, no
normalisation, no products.  Both sides receive exactly the same arrays.
"""
from .rng import stream_rng, for_chunks
from .graphs import erdos_renyi, rmat, chung_lu, relabel, star, ring, directed_rmat
from .dense import uniform_features, normal_features, labels, glorot_weights
from .configs import CONFIGS, make_graph, make_model_inputs, scaled

__all__ = [
    "stream_rng", "for_chunks", "erdos_renyi", "rmat", "chung_lu", "relabel", "star", "ring",
    "directed_rmat", "uniform_features", "normal_features", "labels", "glorot_weights",
    "CONFIGS", "make_graph", "make_model_inputs", "scaled",
]
