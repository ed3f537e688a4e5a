"""Counter-based random streams.

Every array is drawn in fixed-size chunks; chunk ``c`` of stream ``s`` under seed
``seed`` uses its own Philox generator keyed by ``(seed, s, c)``.  The result is
therefore independent of how many threads draw the chunks.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 1 << 20  # elements (edges, or matrix rows x cols rounded to rows) per chunk

# stream ids: one per kind of array, so arrays are independent of one another
STREAM_EDGES = 1
STREAM_PERM = 2
STREAM_FEATURES = 3
STREAM_LABELS = 4
STREAM_WEIGHTS = 5


def stream_rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    key = [np.uint64(seed), (np.uint64(stream) << np.uint64(40)) | np.uint64(chunk)]
    return np.random.Generator(np.random.Philox(key=key))


def n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def for_chunks(total: int, fn, chunk: int = CHUNK):
    """Call ``fn(chunk_index, start, stop)`` for each chunk of ``range(total)``, on a thread
    pool, and return the list of results in chunk order."""
    spans = [(c, s, min(s + chunk, total)) for c, s in enumerate(range(0, total, chunk))]
    if len(spans) <= 1:
        return [fn(*sp) for sp in spans]
    with ThreadPoolExecutor(max_workers=n_workers()) as ex:
        return list(ex.map(lambda sp: fn(*sp), spans))
