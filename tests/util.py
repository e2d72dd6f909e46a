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


def row_rel_max(G: np.ndarray, O: np.ndarray) -> float:
    """Largest per-row relative Frobenius error (rows of a 2-D tensor); one wrong row among thousands does not move
    the norm over the whole tensor, but it does move its own row's."""
    G, O = np.asarray(G, dtype=np.float64), np.asarray(O, dtype=np.float64)
    assert G.shape == O.shape and G.ndim == 2, (G.shape, O.shape)
    if O.size == 0:
        return 0.0
    if not np.all(np.isfinite(G)):
        return float("inf")
    num = np.linalg.norm(G - O, axis=1)
    den = np.linalg.norm(O, axis=1)
    if np.any((den == 0.0) & (num != 0.0)):
        return float("inf")
    return float(np.max(num / np.where(den == 0.0, 1.0, den)))


ELEM_EPS = {"bf16": 2.0 ** -8, "f32": 2.0 ** -20}


def elem_excess(G: np.ndarray, O: np.ndarray, dtype: str, c: float = 4.0) -> float:
    """Per-element bound for the small tensors (S, dS, dA_i, dB_i):  |G - O| <= c eps (|O| + rms), c = 4, eps = 2^-8 for
    bf16 results and 2^-20 for fp32 results.  Where it comes from (bf16): the output rounding is at most 2^-9 |O|; the
    rounded intermediates (dS feeds dA_i, S feeds dB_i, each element off by up to 2^-9 of itself) add a random error
    whose standard deviation is about 2^-9 / sqrt(3) of the tensor's rms; together the observed error has a standard
    deviation of 1.6e-3 .. 2.4e-3 rms, so c eps rms = 1.6e-2 rms is 6.5 or more standard deviations.  rms = the larger of
    the element's row rms and the whole tensor's rms (a row can be a single element).  Returns max |G - O| / bound:
    <= 1 passes.  A single element that misses a term, a row or a chunk is off by the order of the rms itself."""
    G, O = np.asarray(G, dtype=np.float64), np.asarray(O, dtype=np.float64)
    assert G.shape == O.shape, (G.shape, O.shape)
    if O.size == 0:
        return 0.0
    if not np.all(np.isfinite(G)):
        return float("inf")
    O2 = O.reshape(O.shape[0], -1) if O.ndim > 1 else O.reshape(1, -1)
    G2 = G.reshape(O2.shape)
    rms_all = float(np.sqrt(np.mean(O2 * O2)))
    rms_row = np.sqrt(np.mean(O2 * O2, axis=1, keepdims=True))
    bound = c * ELEM_EPS[dtype] * (np.abs(O2) + np.maximum(rms_row, rms_all))
    diff = np.abs(G2 - O2)
    if np.any((bound == 0.0) & (diff != 0.0)):
        return float("inf")
    return float(np.max(diff / np.where(bound == 0.0, 1.0, bound)))


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
