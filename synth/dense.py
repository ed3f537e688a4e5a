"""Dense inputs: feature matrices, labels and initial weights (all float32 / int32)."""
from __future__ import annotations

import numpy as np

from .rng import CHUNK, STREAM_FEATURES, STREAM_LABELS, STREAM_WEIGHTS, for_chunks, stream_rng


def _rows_per_chunk(f: int) -> int:
    return max(1, CHUNK // max(1, f))


def uniform_features(n: int, f: int, seed: int = 0, stream: int = STREAM_FEATURES) -> np.ndarray:
    """n x f float32, entries uniform in [-1, 1)."""
    out = np.empty((n, f), np.float32)

    def draw(c, s, e):
        g = stream_rng(seed, stream, c)
        out[s:e] = g.random((e - s, f), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    for_chunks(n, draw, _rows_per_chunk(f))
    return out


def normal_features(n: int, f: int, seed: int = 0, stream: int = STREAM_FEATURES) -> np.ndarray:
    """n x f float32, entries standard normal."""
    out = np.empty((n, f), np.float32)

    def draw(c, s, e):
        g = stream_rng(seed, stream, c)
        out[s:e] = g.standard_normal((e - s, f), dtype=np.float32)
    for_chunks(n, draw, _rows_per_chunk(f))
    return out


def labels(n: int, n_classes: int, seed: int = 0) -> np.ndarray:
    """n int32 labels uniform in [0, n_classes)."""
    out = np.empty(n, np.int32)

    def draw(c, s, e):
        g = stream_rng(seed, STREAM_LABELS, c)
        out[s:e] = g.integers(0, n_classes, size=e - s, dtype=np.int64).astype(np.int32)
    for_chunks(n, draw)
    return out


def glorot_weights(dims, seed: int = 0):
    """One ``dims[l] x dims[l+1]`` float32 matrix per layer, uniform in +-sqrt(6/(fan_in+fan_out))."""
    ws = []
    for l in range(len(dims) - 1):
        fi, fo = int(dims[l]), int(dims[l + 1])
        g = stream_rng(seed, STREAM_WEIGHTS, l)
        lim = np.sqrt(6.0 / (fi + fo))
        ws.append(((g.random((fi, fo)) * 2.0 - 1.0) * lim).astype(np.float32))
    return ws
