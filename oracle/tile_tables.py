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


NARROW_MAX_RANK = 64      # adapters with a larger rank form the wide rank class


def wgrad_chunks(offsets: Sequence[int], ranks: Sequence[int], chunk_rows: int, chunk_rows_wide: int) -> List[Tuple[int, int, int, int]]:
    """Token chunks the weight-gradient reductions dA_i = X_i^T dS_i, dB_i = s_i S_i^T dY_i are split into (Sec. 5.1:
    one grouped launch reduces every adapter's tokens; App. A.1: work items come from a table built from the
    per-adapter offsets): entries (adapter, chunk index within the adapter, first global row, rows).  Adapters of the
    narrow rank class (rank <= 64) are cut every `chunk_rows` tokens, the others every `chunk_rows_wide`.

    Launch order = order of the table: the wide class first (its items run longest and go through a kernel build of
    their own), then the narrow class; inside a class by decreasing cost rows x (64 + rank) -- the stream of X / dY
    rows dominates, the MFMA work grows with the rank -- so that long items start first and short ones fill the
    compute units as they drain; equal costs keep the canonical order (adapter ascending, chunk ascending)."""
    canon = []
    for i in range(len(offsets) - 1):
        r = ranks[i]
        if offsets[i + 1] <= offsets[i] or r <= 0:
            continue
        per = chunk_rows if r <= NARROW_MAX_RANK else chunk_rows_wide
        c, row = 0, offsets[i]
        while row < offsets[i + 1]:
            rows = min(per, offsets[i + 1] - row)
            canon.append((i, c, row, rows))
            row += rows
            c += 1
    order = []
    for pos, en in enumerate(canon):
        narrow = 1 if ranks[en[0]] <= NARROW_MAX_RANK else 0
        cost = en[3] * (64 + ranks[en[0]])
        order.append((narrow, -cost, pos, en))
    order.sort()
    return [en for _, _, _, en in order]


def class_blocks(offsets: Sequence[int], ranks: Sequence[int], block_rows: int, block_rows_wide: int) -> List[Tuple[int, int, int, int]]:
    """The LoRA blocks in the order the grouped kernels walk them (App. A.1: one table entry per (adapter, block);
    the order of the entries is free): blocks of the wide rank class (rank > 64) first -- they take longest and go
    through a kernel build of their own --, then the narrow class, canonical order inside a class.  Wide adapters
    are cut every `block_rows_wide` rows, narrow ones every `block_rows`."""
    wide, narrow = [], []
    for i in range(len(offsets) - 1):
        r = ranks[i]
        if offsets[i + 1] <= offsets[i] or r <= 0:
            continue
        per = block_rows if r <= NARROW_MAX_RANK else block_rows_wide
        b, row = 0, offsets[i]
        while row < offsets[i + 1]:
            rows = min(per, offsets[i + 1] - row)
            (narrow if r <= NARROW_MAX_RANK else wide).append((i, b, row, rows))
            row += rows
            b += 1
    return wide + narrow


def wgrad_chunk_rows(offsets: Sequence[int], ranks: Sequence[int], k: int, n: int, num_cus: int,
                     panel_cols: int, min_chunk_rows: int) -> Tuple[int, int]:
    """Token chunk of the weight-gradient work items, (narrow class, wide class): the balancing rule for
    heterogeneous segment lengths.  A work item is (token chunk of one adapter, panel of `panel_cols` columns of X or
    dY), so one launch has sum_i ceil(T_i / chunk) x (ceil(k / panel_cols) + ceil(n / panel_cols)) items.  The chunk
    is the largest power of two, at most 2^30, for which the launch has at least two items per compute unit, and
    never below `min_chunk_rows` (whole segments -- no partial sums at all -- whenever they already give enough
    items).  A plan that holds adapters of both rank classes runs one launch per class, and the rule is applied to
    each launch by itself; otherwise both values are the one chunk of the single launch."""
    panels = -(-k // panel_cols) + -(-n // panel_cols)
    live = [(offsets[i + 1] - offsets[i], ranks[i]) for i in range(len(ranks)) if offsets[i + 1] > offsets[i] and ranks[i] > 0]

    def choose(lens):
        chunk = 1 << 30
        while chunk > min_chunk_rows:
            items = sum(-(-t // chunk) for t in lens) * panels
            if items >= 2 * num_cus:
                break
            chunk //= 2
        return chunk

    narrow = [t for t, r in live if r <= NARROW_MAX_RANK]
    wide = [t for t, r in live if r > NARROW_MAX_RANK]
    if narrow and wide:
        return choose(narrow), choose(wide)
    c = choose(narrow + wide)
    return c, c


def gemm_band_order(offsets: Sequence[int], ranks: Sequence[int], tile_rows: int, band_tiles: int) -> List[Tuple[int, int, int, int]]:
    """Launch order of the fused GEMM's row bands: (band, first row tile, row tiles, cost).  A band is `band_tiles`
    consecutive row tiles of the flat buffer (the last band may have fewer).  The fused GEMM adds, per output tile, one
    masked rank-extension pass per 64 ranks of every adapter that owns rows of the tile (found here by scanning the
    rows); the cost of a band is the number of such passes over its row tiles.  Full bands go first by decreasing
    cost, equal costs in band order; a shorter last band stays last."""
    T = offsets[-1]
    n_tiles = -(-T // tile_rows)
    bands = []
    for b in range(-(-n_tiles // band_tiles)):
        t0 = b * band_tiles
        nt = min(band_tiles, n_tiles - t0)
        cost = 0
        for t in range(t0, t0 + nt):
            owners = sorted({owner_linear(offsets, row) for row in range(t * tile_rows, min(T, (t + 1) * tile_rows))})
            cost += sum(-(-ranks[i] // 64) for i in owners if ranks[i] > 0)
        bands.append((b, t0, nt, cost))
    full = [e for e in bands if e[2] == band_tiles]
    part = [e for e in bands if e[2] != band_tiles]
    full.sort(key=lambda e: (-e[3], e[0]))
    return full + part
