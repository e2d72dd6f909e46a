"""Pins for the bookkeeping oracle (App. A.1: (adapter, block) schedule table over
per-adapter offsets, boundary blocks masked, no padding)."""
import numpy as np

from oracle import tile_tables as tt


def test_row_blocks_cover_every_row_exactly_once_and_count_matches():
    rng = np.random.default_rng(0)
    for trial in range(50):
        N = int(rng.integers(1, 9))
        lens = [int(x) for x in rng.integers(0, 300, size=N)]
        ranks = [int(x) for x in rng.choice([0, 1, 4, 8, 33, 128], size=N)]
        off = [0] + list(np.cumsum(lens))
        bm = int(rng.choice([1, 16, 64, 128]))
        tab = tt.row_blocks(off, ranks, bm)
        assert len(tab) == sum(-(-t // bm) for t, r in zip(lens, ranks) if r > 0)
        seen = np.zeros(off[-1] + 1, dtype=int)
        for (i, b, row0, rows) in tab:
            assert 1 <= rows <= bm and row0 == off[i] + b * bm
            for t in range(row0, row0 + rows):
                assert tt.owner_linear(off, t) == i
                seen[t] += 1
        for t in range(off[-1]):
            assert seen[t] == (1 if ranks[tt.owner_linear(off, t)] > 0 else 0)
        assert tab == sorted(tab)


def test_worked_example():
    # offsets 0,5,5,12 with block 4: adapter 0 -> rows 0-3, 4; adapter 1 empty; adapter 2 -> 5-8, 9-11
    assert tt.row_blocks([0, 5, 5, 12], [8, 8, 16], 4) == [(0, 0, 0, 4), (0, 1, 4, 1), (2, 0, 5, 4), (2, 1, 9, 3)]
    assert tt.row_blocks([0, 5, 5, 12], [0, 8, 16], 4) == [(2, 0, 5, 4), (2, 1, 9, 3)]
    assert tt.gemm_row_tiles([0, 5, 5, 12], 8) == [(0, 8, 0, 3), (8, 4, 2, 3)]
    assert tt.gemm_row_tiles([0, 0, 3], 8) == [(0, 3, 1, 2)]
    assert tt.gemm_row_tiles([0, 0], 8) == []


def test_gemm_row_tiles_segment_ranges():
    rng = np.random.default_rng(1)
    for trial in range(30):
        N = int(rng.integers(1, 7))
        lens = [int(x) for x in rng.integers(0, 200, size=N)]
        off = [0] + list(np.cumsum(lens))
        tiles = tt.gemm_row_tiles(off, 64)
        assert sum(r for (_, r, _, _) in tiles) == off[-1]
        for (row0, rows, lo, hi) in tiles:
            assert off[lo] <= row0 < off[lo + 1]
            assert off[hi - 1] <= row0 + rows - 1 < off[hi]
