"""Shared helpers of the GPU parity tests: sampling of rows/columns and the error metric."""
from __future__ import annotations

import numpy as np


def rel_fro(G: np.ndarray, O: np.ndarray) -> float:
    """||G - O||_F / ||O||_F in fp64; a zero oracle tensor requires an exactly zero result."""
    G, O = np.asarray(G, dtype=np.float64), np.asarray(O, dtype=np.float64)
    assert G.shape == O.shape, (G.shape, O.shape)
    if O.size == 0:
        return 0.0
    if not np.all(np.isfinite(G)):
        return float("inf")
    den = np.linalg.norm(O)
    num = np.linalg.norm(G - O)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def sample_rows(offsets, T, tile_rows, count, seed):
    """First and last row of every segment, rows on both sides of every tile boundary,
    and random rows up to `count`."""
    rows = set()
    for i in range(len(offsets) - 1):
        if offsets[i + 1] > offsets[i]:
            rows.update([offsets[i], offsets[i + 1] - 1])
    for b in range(tile_rows, T, tile_rows):
        rows.update([b - 1, b])
    if T:
        rows.update([0, T - 1])
    rng = np.random.default_rng(seed)
    if T and len(rows) < count:
        rows.update(int(x) for x in rng.integers(0, T, size=count - len(rows)))
    return np.array(sorted(r for r in rows if 0 <= r < T), dtype=np.int64)


def sample_cols(n, tile_cols, count, seed):
    cols = {0, n - 1}
    for b in range(tile_cols, n, tile_cols):
        cols.update([b - 1, b])
    rng = np.random.default_rng(seed + 1)
    if len(cols) < count:
        cols.update(int(x) for x in rng.integers(0, n, size=count - len(cols)))
    return np.array(sorted(c for c in cols if 0 <= c < n), dtype=np.int64)
