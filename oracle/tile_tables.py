"""Bookkeeping oracle -- TEST INFRASTRUCTURE ONLY.

Brute-force statements of the integer tables a multi-LoRA plan needs (paper App. A.1,
"schedule-driven dispatch": a table of (adapter_idx, block_idx) pairs, each block
mapped to a token range through per-adapter start/end offsets, boundary blocks masked
at the segment end, no padding of the token buffer).  Pure Python loops, no clever
arithmetic: every row's owner is found by a linear scan of the offsets.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def owner_linear(offsets: Sequence[int], t: int) -> int:
    """Adapter that owns global row t: the i with off[i] <= t < off[i+1] (linear scan)."""
    for i in range(len(offsets) - 1):
        if offsets[i] <= t < offsets[i + 1]:
            return i
    raise ValueError(f"row {t} is outside every segment")


def row_blocks(offsets: Sequence[int], ranks: Sequence[int], block_rows: int) -> List[Tuple[int, int, int, int]]:
    """Canonical LoRA block table: for adapter i ascending, block b ascending,
    (i, b, first global row, number of rows).  Adapters with no tokens or rank 0
    have no LoRA work and contribute no entries."""
    out = []
    for i in range(len(offsets) - 1):
        Ti = offsets[i + 1] - offsets[i]
        if Ti <= 0 or ranks[i] <= 0:
            continue
        b = 0
        row = offsets[i]
        while row < offsets[i + 1]:
            rows = min(block_rows, offsets[i + 1] - row)
            out.append((i, b, row, rows))
            row += rows
            b += 1
    return out


def gemm_row_tiles(offsets: Sequence[int], tile_rows: int) -> List[Tuple[int, int, int, int]]:
    """Row tiles of the flat [T, .] buffer (not aligned to segments) with the range of
    adapters whose segments they touch: (first row, rows, first adapter, last adapter + 1).
    Found by scanning every row of the tile."""
    T = offsets[-1]
    out = []
    row0 = 0
    while row0 < T:
        rows = min(tile_rows, T - row0)
        owners = [owner_linear(offsets, t) for t in range(row0, row0 + rows)]
        out.append((row0, rows, min(owners), max(owners) + 1))
        row0 += rows
    return out
