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


def test_wgrad_chunks_worked_example():
    # adapter 0: 5 tokens rank 8 (narrow, chunk 4) -> chunks of 4 and 1; adapter 1 has no tokens; adapter 2: 7 tokens
    # rank 128 (wide, chunk 3) -> 3, 3, 1; adapter 3: rank 0, no work.  Costs rows x (64 + rank): wide 576, 576, 192;
    # narrow 288, 72.  Wide class first, each class by decreasing cost, ties in canonical order.
    got = tt.wgrad_chunks([0, 5, 5, 12, 20], [8, 8, 128, 0], 4, 3)
    assert got == [(2, 0, 5, 3), (2, 1, 8, 3), (2, 2, 11, 1), (0, 0, 0, 4), (0, 1, 4, 1)]
    # one class only, one chunk size: a longer low-rank chunk can cost more than a shorter high-rank one
    got = tt.wgrad_chunks([0, 10, 14], [4, 64], 8, 8)
    assert got == [(0, 0, 0, 8), (1, 0, 10, 4), (0, 1, 8, 2)]      # 8*68 = 544 > 4*128 = 512 > 2*68 = 136
    assert tt.wgrad_chunks([0, 0], [8], 4, 4) == []


def test_wgrad_chunks_cover_every_ranked_row_exactly_once_and_are_ordered():
    rng = np.random.default_rng(2)
    for trial in range(60):
        N = int(rng.integers(1, 10))
        lens = [int(x) for x in rng.integers(0, 400, size=N)]
        ranks = [int(x) for x in rng.choice([0, 1, 4, 8, 33, 64, 65, 128], size=N)]
        off = [0] + [int(x) for x in np.cumsum(lens)]
        cn, cw = int(rng.choice([1, 16, 100, 512])), int(rng.choice([1, 7, 64, 512]))
        tab = tt.wgrad_chunks(off, ranks, cn, cw)
        seen = np.zeros(off[-1] + 1, dtype=int)
        per_adapter = {}
        for (i, c, row0, rows) in tab:
            per = cn if ranks[i] <= 64 else cw
            assert 1 <= rows <= per and row0 == off[i] + c * per and row0 + rows <= off[i + 1]
            for t in range(row0, row0 + rows):
                assert tt.owner_linear(off, t) == i
                seen[t] += 1
            per_adapter.setdefault(i, []).append(c)
        for t in range(off[-1]):
            assert seen[t] == (1 if ranks[tt.owner_linear(off, t)] > 0 else 0)
        for i, cs in per_adapter.items():                     # chunk indices 0..count-1, each once
            per = cn if ranks[i] <= 64 else cw
            assert sorted(cs) == list(range(-(-lens[i] // per)))
        # order: no narrow entry before a wide one; costs never increase inside a class; equal costs in canonical order
        cls = [0 if ranks[en[0]] > 64 else 1 for en in tab]
        assert cls == sorted(cls)
        for a, b in zip(tab, tab[1:]):
            if (ranks[a[0]] > 64) != (ranks[b[0]] > 64):
                continue
            ca, cb = a[3] * (64 + ranks[a[0]]), b[3] * (64 + ranks[b[0]])
            assert ca > cb or (ca == cb and (a[0], a[1]) < (b[0], b[1]))


def test_class_blocks_are_the_row_blocks_wide_class_first():
    assert tt.class_blocks([0, 5, 5, 12, 14], [8, 8, 100, 16], 4, 4) == \
        [(2, 0, 5, 4), (2, 1, 9, 3), (0, 0, 0, 4), (0, 1, 4, 1), (3, 0, 12, 2)]
    # wide adapters may be cut differently
    assert tt.class_blocks([0, 5, 12], [8, 100], 4, 8) == [(1, 0, 5, 7), (0, 0, 0, 4), (0, 1, 4, 1)]
    rng = np.random.default_rng(3)
    for trial in range(40):
        N = int(rng.integers(1, 9))
        lens = [int(x) for x in rng.integers(0, 300, size=N)]
        ranks = [int(x) for x in rng.choice([0, 4, 64, 65, 128], size=N)]
        off = [0] + [int(x) for x in np.cumsum(lens)]
        tab = tt.class_blocks(off, ranks, 64, 64)
        assert sorted(tab) == tt.row_blocks(off, ranks, 64)               # same entries
        cls = [0 if ranks[e[0]] > 64 else 1 for e in tab]
        assert cls == sorted(cls)
        wide, narrow = [e for e in tab if ranks[e[0]] > 64], [e for e in tab if ranks[e[0]] <= 64]
        assert wide == sorted(wide) and narrow == sorted(narrow)


def test_wgrad_chunk_rows_rule():
    # 8 x 2048 tokens, 4096 x 4096, 256 CUs, 128-column panels: 64 panels x 8 whole segments = 512 items = 2 per CU
    off = [2048 * i for i in range(9)]
    assert tt.wgrad_chunk_rows(off, [8] * 8, 4096, 4096, 256, 128, 512) == (1 << 30, 1 << 30)
    # 7 such segments give 448 items: the chunk is halved until 2048 still gives 448, 1024 gives 896 >= 512
    assert tt.wgrad_chunk_rows(off[:8], [8] * 7, 4096, 4096, 256, 128, 512) == (1024, 1024)
    # one short segment through a narrow layer never reaches two items per CU: the minimum chunk
    assert tt.wgrad_chunk_rows([0, 3000], [16], 256, 256, 256, 128, 512) == (512, 512)
    # both rank classes present: each launch balanced by itself (6 narrow segments: 384 items whole, 768 at 1024;
    # 2 wide ones: 128 whole, 256 at 1024, 512 at 512)
    assert tt.wgrad_chunk_rows(off, [8] * 6 + [128] * 2, 4096, 4096, 256, 128, 512) == (1024, 512)
    # adapters without tokens or without rank do not count (here nothing is live: no items at any chunk, the floor)
    assert tt.wgrad_chunk_rows([0, 0, 2048], [8, 0], 4096, 4096, 256, 128, 512) == (512, 512)
    assert tt.wgrad_chunk_rows([0, 0, 100] + [100 + 2048 * i for i in range(1, 9)], [8, 0] + [8] * 8,
                               4096, 4096, 256, 128, 512) == (1 << 30, 1 << 30)
    rng = np.random.default_rng(4)
    for trial in range(40):
        N = int(rng.integers(1, 20))
        lens = [int(x) for x in rng.integers(0, 5000, size=N)]
        ranks = [int(x) for x in rng.choice([0, 8, 64, 128], size=N)]
        off = [0] + [int(x) for x in np.cumsum(lens)]
        k, n, cus = int(rng.choice([64, 1024, 4096])), int(rng.choice([64, 4096, 14336])), 256
        panels = -(-k // 128) + -(-n // 128)
        cn, cw = tt.wgrad_chunk_rows(off, ranks, k, n, cus, 128, 512)
        live_n = [t for t, r in zip(lens, ranks) if t > 0 and 0 < r <= 64]
        live_w = [t for t, r in zip(lens, ranks) if t > 0 and r > 64]
        groups = [(cn, live_n), (cw, live_w)] if live_n and live_w else [(cn, live_n + live_w)]
        assert (live_n and live_w) or cn == cw
        for c, ls in groups:
            items = lambda ch: sum(-(-t // ch) for t in ls) * panels
            assert c & (c - 1) == 0 and 512 <= c <= 1 << 30
            assert items(c) >= 2 * cus or c == 512                         # enough items, or the floor
            assert c == 1 << 30 or items(2 * c) < 2 * cus                 # and no larger chunk would have done


def test_gemm_band_order_worked_example_and_properties():
    # tiles of 4 rows, bands of 2 tiles; T = 22 -> tiles 0..5 (the last of 2 rows), bands (0,1) (2,3) (4,5): all full
    # adapters: rows 0-2 rank 8, rows 3-9 rank 128, rows 10-21 rank 0
    # tile 0 (rows 0-3): adapters 0, 1 -> 1 + 2 = 3 passes; tile 1 (4-7): 2; tile 2 (8-11): adapter 1 -> 2 (adapter 2 has no rank);
    # tiles 3, 4, 5: 0
    assert tt.gemm_band_order([0, 3, 10, 22], [8, 128, 0], 4, 2) == [(0, 0, 2, 5), (1, 2, 2, 2), (2, 4, 2, 0)]
    # costs increasing down the buffer: the order is reversed; a shorter last band stays last whatever it costs
    assert tt.gemm_band_order([0, 8, 16, 20], [0, 64, 128], 4, 2) == [(1, 2, 2, 2), (0, 0, 2, 0), (2, 4, 1, 2)]
    assert tt.gemm_band_order([0, 0], [8], 4, 2) == []
    rng = np.random.default_rng(5)
    for trial in range(30):
        N = int(rng.integers(1, 8))
        lens = [int(x) for x in rng.integers(0, 120, size=N)]
        ranks = [int(x) for x in rng.choice([0, 8, 64, 65, 128], size=N)]
        off = [0] + [int(x) for x in np.cumsum(lens)]
        order = tt.gemm_band_order(off, ranks, 16, 4)
        n_tiles = -(-off[-1] // 16)
        assert sorted(e[0] for e in order) == list(range(-(-n_tiles // 4)))          # a permutation of the bands
        assert sum(e[2] for e in order) == n_tiles
        for e in order[:-1]:
            assert e[2] == 4
        full = [e for e in order if e[2] == 4]
        for a, b in zip(full, full[1:]):
            assert a[3] > b[3] or (a[3] == b[3] and a[0] < b[0])
        # total cost = sum over (tile, adapter that owns rows of it) of ceil(rank / 64), counted from the tile table
        tiles = tt.gemm_row_tiles(off, 16)
        want = 0
        for (row0, rows, lo, hi) in tiles:
            for i in range(lo, hi):
                if ranks[i] > 0 and min(off[i + 1], row0 + rows) > max(off[i], row0):
                    want += -(-ranks[i] // 64)
        assert sum(e[3] for e in order) == want
