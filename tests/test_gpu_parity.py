"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element on
the same seeded inputs.  Tolerances: relative Frobenius error <= 1e-2 for bf16 tensors and
<= 1e-5 for fp32 runs; integer bookkeeping bit-exact."""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from oracle import tile_tables as tt
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_device, to_host
from util import elem_excess, rel_fro, row_rel_max, sample_cols, sample_rows

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-5}


def check_full(w, tol=None, label=""):
    """Run fwd+bwd on the GPU and compare every output with the full oracle."""
    tol = TOL[w.dtype] if tol is None else tol
    print(f"[case] {label or w.name} dtype={w.dtype} T={w.T} k={w.k} n={w.n} ranks={w.ranks} lens={w.seg_lens}", flush=True)
    dl = DeviceLayer(w)
    dl.forward()
    dl.backward()
    dl.sync()
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    Yg, dXg = to_host(dl.Y), to_host(dl.dX)
    errs = {"Y": rel_fro(Yg, fw.Y), "dX": rel_fro(dXg, bw.dX)}
    # every row by itself as well (the norm over the whole tensor hides a single wrong row)
    errs["Y_row_max"], errs["dX_row_max"] = row_rel_max(Yg, fw.Y), row_rel_max(dXg, bw.dX)
    S, dS = dl.S_list(), dl.dS_list()
    elem = {}
    for i in range(w.N):
        got = {"S": S[i], "dS": dS[i], "dA": to_host(dl.dA[i]), "dB": to_host(dl.dB[i])}
        want = {"S": fw.S[i], "dS": bw.dS[i], "dA": bw.dA[i], "dB": bw.dB[i]}
        for name in got:
            errs[f"{name}{i}"] = rel_fro(got[name], want[name])
            elem[f"{name}{i}"] = elem_excess(got[name], want[name], w.dtype)     # and every element by itself
    worst = max(errs.items(), key=lambda kv: kv[1])
    worst_e = max(elem.items(), key=lambda kv: kv[1]) if elem else ("-", 0.0)
    print(f"        worst {worst[0]} = {worst[1]:.3e}; worst element {worst_e[0]} at {worst_e[1]:.2f} of its bound", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    bad.update({k + "_elem": v for k, v in elem.items() if not v <= 1.0})
    assert not bad, bad
    return dl, fw, bw


# ---- bookkeeping ------------------------------------------------------------------------
def test_plan_tables_bit_exact():
    rng = np.random.default_rng(0)
    cases = [([0, 5, 5, 12], [8, 8, 16]), ([0, 0], [4]), ([0, 300], [0]),
             ([0, 3000, 7000, 7100, 30000], [128, 8, 100, 64])]      # many row bands with unequal rank-extension work
    for _ in range(12):
        N = int(rng.integers(1, 40))
        lens = [int(x) for x in rng.integers(0, 3000, size=N)]
        ranks = [int(x) for x in rng.choice([0, 1, 4, 8, 33, 64, 128], size=N)]
        cases.append(([0] + [int(x) for x in np.cumsum(lens)], ranks))
    shapes = [(64, 64), (4096, 4096), (1024, 14336), (256, 128)]
    for c, (off, ranks) in enumerate(cases):
        T = off[-1]
        k, n = shapes[c % len(shapes)]            # the layer shape enters the token chunk through the panel count
        plan = ml.Plan(ml.BF16, T, k, n, ranks, [1.0] * len(ranks), off)
        geo = plan.geometry()
        assert plan.dump(ml.TABLE_ROW_BLOCKS) == tt.row_blocks(off, ranks, geo[ml.GEO_BLOCK_ROWS])
        assert plan.dump(ml.TABLE_CLASS_BLOCKS) == tt.class_blocks(off, ranks, geo[ml.GEO_BLOCK_ROWS], geo[ml.GEO_BLOCK_ROWS_WIDE])
        # the token chunks the device-side scheduler chose, and the item table it built and ordered from them
        cn, cw = geo[ml.GEO_WGRAD_CHUNK_ROWS], geo[ml.GEO_WGRAD_CHUNK_ROWS_WIDE]
        assert (cn, cw) == tt.wgrad_chunk_rows(off, ranks, k, n, geo[ml.GEO_NUM_CUS], geo[ml.GEO_WGRAD_PANEL_COLS],
                                               geo[ml.GEO_WGRAD_MIN_CHUNK_ROWS])
        assert plan.dump(ml.TABLE_WGRAD_CHUNKS) == tt.wgrad_chunks(off, ranks, cn, cw)
        assert plan.dump(ml.TABLE_GEMM_ROW_TILES) == tt.gemm_row_tiles(off, geo[ml.GEO_GEMM_TILE_ROWS])
        assert plan.dump(ml.TABLE_GEMM_BAND_ORDER) == tt.gemm_band_order(off, ranks, geo[ml.GEO_GEMM_TILE_ROWS],
                                                                         geo[ml.GEO_GEMM_BAND_TILES])
        lens = [off[i + 1] - off[i] for i in range(len(ranks))]
        assert plan.R1 == sum(t * r for t, r in zip(lens, ranks))
        plan.destroy()


# ---- config 1: tiny fp32 ------------------------------------------------------------------
def test_config_tiny_fp32_full_oracle():
    check_full(wl.config(0))


def test_fp32_ragged_small():
    w = wl.small_case(seed=21, dtype="f32", k=200, n=136, ranks=(4, 16, 0, 33, 128, 8),
                      seg_lens=(129, 1, 70, 257, 65, 0), b_sigma=0.3)
    check_full(w)


# ---- bf16 MFMA path: ragged small cases spanning several tiles ------------------------------
@pytest.mark.parametrize("seed,k,n,ranks,lens", [
    (31, 512, 768, (4, 16, 0, 33, 128, 8), (129, 1, 70, 257, 300, 0)),
    (32, 320, 264, (1, 3, 12, 100, 64), (63, 257, 5, 200, 1100)),     # k, n not multiples of the tile
    (33, 1024, 512, (8, 8, 16, 64), (256, 256, 512, 1300)),           # a segment split over wgrad chunks
    (34, 64, 8, (128,), (2100,)),
    (37, 200, 136, (8, 128, 24), (100, 333, 64)),                     # both contractions end in a partial 64-wide tile
    (38, 256, 512, (96, 40), (190, 70)),                              # ranks above 64 select the wide-rank kernels
])
def test_bf16_ragged_small(seed, k, n, ranks, lens):
    w = wl.small_case(seed=seed, dtype="bf16", k=k, n=n, ranks=ranks, seg_lens=lens,
                      scales=[2.0, 0.5, 1.0, 16.0 / 33.0, 0.125, 3.0][: len(ranks)], b_sigma=0.3)
    check_full(w)


@pytest.mark.parametrize("k,n", [(64, 128), (128, 64), (192, 256), (256, 192), (40, 72), (72, 40), (96, 520), (520, 96)])
def test_bf16_contraction_lengths_around_the_two_stage_pipeline(k, n):
    # the fused GEMM keeps two tiles in LDS and loads two tiles ahead: contractions of 0, 1, 2, 3, 4 and 8 whole
    # 64-wide tiles, with and without a partial tile, exercise its prologue, steady state and drain (forward
    # contracts over k, backward over n); 300 rows = one full 256-row tile and a partial one
    w = wl.small_case(seed=70 + k % 7 + n % 5, dtype="bf16", k=k, n=n, ranks=(8, 40), seg_lens=(300, 45),
                      scales=(2.0, 0.5), b_sigma=0.3)
    check_full(w)


@pytest.mark.parametrize("k,n", [(320, 264), (128, 576)])
def test_tiles_owned_by_one_adapter_take_every_rank_through_the_direct_loads(k, n):
    """Segments that are multiples of the 256-row GEMM tile: every tile belongs to one adapter, so its rank extension
    fetches S_i / B_i (dS_i / A_i) by direct loads.  The ranks cover every case of that path: one and two 64-rank passes,
    ranks that are multiples of 32 (nothing to zero), ranks that end 8, 16 or 24 short of a 32-wide MFMA step in the first
    and in the second half of a pass, rank 0 (no pass), and a last segment that ends inside a tile (rows past T).  The
    scales are not powers of two, so a rounding of s_i S_i to bf16 would show in the per-element bound."""
    ranks = (8, 24, 40, 56, 72, 104, 120, 128, 64, 32, 0, 16)
    lens = (256, 512, 256, 256, 512, 256, 256, 256, 256, 512, 256, 256 + 77)
    scales = [16.0 / 33.0, 3.0, 0.3, 1.7, 16.0 / 72.0, 0.77, 1.0, 2.0, 0.9, 1.1, 5.0, 0.6]
    w = wl.small_case(seed=81 + k % 3, dtype="bf16", k=k, n=n, ranks=ranks, seg_lens=lens, scales=scales, b_sigma=0.3)
    check_full(w)


def test_bf16_odd_widths_use_fma_kernels():
    w = wl.small_case(seed=35, dtype="bf16", k=100, n=52, ranks=(4, 7, 0, 16), seg_lens=(33, 64, 10, 70),
                      scales=(2.0, 0.5, 1.0, 1.5), b_sigma=0.3)
    dl, _, _ = check_full(w)
    assert dl.plan.geometry()[ml.GEO_USES_MFMA] == 0


def test_bf16_aligned_uses_mfma_kernels():
    w = wl.small_case(seed=36, dtype="bf16", k=128, n=128, ranks=(8,), seg_lens=(100,), scales=(1.0,))
    dl, _, _ = check_full(w)
    assert dl.plan.geometry()[ml.GEO_USES_MFMA] == 1


def test_many_adapters_span_several_pointer_batches():
    rng = np.random.default_rng(7)
    N = 45
    ranks = [int(x) for x in rng.choice([0, 4, 8, 16, 24], size=N)]
    lens = [int(x) for x in rng.integers(0, 60, size=N)]
    w = wl.make_workload("many", "bf16", 128, 192, ranks, lens, [float(x) for x in rng.choice([0.5, 1.0, 2.0], size=N)],
                         seed=39, b_sigma=0.3)
    check_full(w)


def test_all_segments_empty():
    for dtype in ("bf16", "f32"):
        w = wl.make_workload("empty", dtype, 64, 64, [8, 16], [0, 0], [1.0, 2.0], seed=40)
        dl = DeviceLayer(w); dl.forward(); dl.backward(); dl.sync()
        for i in range(2):
            assert torch.all(dl.dA[i] == 0) and torch.all(dl.dB[i] == 0)


# ---- flags -------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,ranks", [("bf16", (4, 16, 0, 40, 8)), ("f32", (4, 16, 0, 40, 8)), ("bf16", (4, 100, 0, 128, 7))])
def test_base_only_and_lora_only_modes(dtype, ranks):
    w = wl.small_case(seed=41, dtype=dtype, k=256, n=392, ranks=ranks, seg_lens=(129, 1, 70, 257, 90),
                      scales=(2.0, 0.5, 1.0, 0.4, 3.0), b_sigma=0.3)
    tol = TOL[dtype]
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets, want_base=True)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    dl = DeviceLayer(w)
    dl.forward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_BASE_ONLY); dl.sync()
    assert rel_fro(to_host(dl.Y), fw.Ybase) <= tol
    dXbase = w.dY.astype(np.float64) @ w.W.astype(np.float64).T
    assert rel_fro(to_host(dl.dX), dXbase) <= tol
    # LoRA-only: Y and dX start at zero, so they end up holding the LoRA terms alone
    dl.Y.zero_(); dl.dX.zero_()
    dl.forward(ml.FLAG_LORA_ONLY); dl.backward(ml.FLAG_LORA_ONLY); dl.sync()
    assert rel_fro(to_host(dl.Y), fw.Y - fw.Ybase) <= tol
    assert rel_fro(to_host(dl.dX), bw.dX - dXbase) <= tol
    for i in range(w.N):
        assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= tol and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= tol
    # LoRA-only on top of a base-only result reproduces the fused result within tolerance
    dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY); dl.sync()
    assert rel_fro(to_host(dl.Y), fw.Y) <= tol


@pytest.mark.parametrize("dtype,lens", [("bf16", (300, 1200, 77, 0)), ("f32", (129, 70, 33, 0))])
def test_gradient_accumulation_flag(dtype, lens):
    # two backward calls with MLORA_FLAG_ACCUM_GRADS on zeroed gradients hold twice the oracle's dA_i, dB_i; dX is
    # overwritten as usual; the 1200-token segment is split over several weight-gradient chunks in the bf16 plan
    w = wl.small_case(seed=64, dtype=dtype, k=256, n=320, ranks=(8, 64, 100, 16), seg_lens=lens,
                      scales=(2.0, 0.25, 1.0, 3.0), b_sigma=0.3)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
    dl = DeviceLayer(w)
    dl.forward()
    for t in dl.dA + dl.dB:
        t.zero_()
    dl.backward(ml.FLAG_ACCUM_GRADS); dl.backward(ml.FLAG_ACCUM_GRADS); dl.sync()
    tol = TOL[dtype]
    assert rel_fro(to_host(dl.dX), bw.dX) <= tol
    for i in range(w.N):
        assert rel_fro(to_host(dl.dA[i]), 2.0 * bw.dA[i]) <= tol, i
        assert rel_fro(to_host(dl.dB[i]), 2.0 * bw.dB[i]) <= tol, i
    dl.backward(); dl.sync()          # without the flag the gradients are overwritten again
    for i in range(w.N):
        assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= tol and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= tol
    with pytest.raises(ml.MultiLoraError) as e:   # the flag belongs to the backward
        dl.forward(ml.FLAG_ACCUM_GRADS)
    assert e.value.status == -9


# ---- degenerate shapes ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_no_adapters_and_no_tokens(dtype):
    w = wl.make_workload("noadapters", dtype, 128, 64, [], [], [], seed=50)
    assert w.T == 0
    dl = DeviceLayer(w); dl.forward(); dl.backward(); dl.sync()           # T = 0, N = 0: nothing to do
    w = wl.make_workload("rank0", dtype, 128, 64, [0], [37], [1.0], seed=51)
    dl, fw, _ = check_full(w)                                                # plain X W
    w = wl.make_workload("emptyseg", dtype, 128, 64, [8, 16], [0, 300], [1.0, 2.0], seed=52)
    dl, _, _ = check_full(w)                                                 # adapter 0 has a rank but no tokens
    assert torch.all(dl.dA[0] == 0) and torch.all(dl.dB[0] == 0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_no_adapters_with_tokens(dtype):
    """N = 0 with T > 0: every row is a plain X W row; the metadata and pointer arrays may be NULL."""
    T, k, n = 300, 128, 192
    ref = wl.make_workload("plain", dtype, k, n, [0], [T], [1.0], seed=54)     # same numbers through a rank-0 adapter
    fw = orc.forward(ref.X, ref.W, ref.A, ref.B, ref.scales, ref.offsets)
    bw = orc.backward(ref.dY, ref.X, ref.W, ref.A, ref.B, ref.scales, ref.offsets)
    dev = torch.device("cuda:0")
    X, W, dY = (to_device(a, dtype, dev) for a in (ref.X, ref.W, ref.dY))
    Y = torch.full((T, n), float("nan"), dtype=X.dtype, device=dev)
    dX = torch.full((T, k), float("nan"), dtype=X.dtype, device=dev)
    plan = ml.Plan(ml.BF16 if dtype == "bf16" else ml.F32, T, k, n, [], None, None)
    assert plan.workspace_bytes() == 0
    ml.multi_lora_fwd(plan, X, W, None, None, Y, None, None)
    ml.multi_lora_bwd(plan, dY, None, W, None, None, None, dX, None, None, None)
    torch.cuda.synchronize()
    assert rel_fro(to_host(Y), fw.Y) <= TOL[dtype] and rel_fro(to_host(dX), bw.dX) <= TOL[dtype]
    plan.destroy()


def test_tall_and_thin_layer():
    """200 000 rows through 64 x 72: many row tiles and row blocks, a single partial column tile, one segment of 150 000
    tokens (its weight gradients are reduced from several chunks), an odd rank and the widest one."""
    w = wl.make_workload("tall", "bf16", 64, 72, [8, 128, 3, 0], [150_000, 30_000, 19_999, 1], [2.0, 0.125, 1.0, 1.0],
                         seed=55, b_sigma=0.3)
    dl, _, _ = check_full(w)
    assert dl.plan.geometry()[ml.GEO_USES_MFMA] == 1


def test_few_tokens_through_a_large_weight():
    """5 tokens through 8192 x 4096 (decode-like shape): one partial row tile, long contraction, 64 weight-gradient panels
    of a 3-token and a 2-token segment."""
    w = wl.make_workload("flat", "bf16", 8192, 4096, [16, 64], [3, 2], [1.0, 0.25], seed=56, b_sigma=0.3)
    check_full(w)


def test_rank_padded_stacked_adapters_equal_true_rank_adapters():
    """The paper's stacked layout (App. A.1: adapters of different ranks zero-padded to r_max in one [Z, k, r_max] /
    [Z, r_max, n] pair of tensors) is served by declaring every adapter with rank r_max and pointing into the stacks: the
    padding columns / rows are zero, so Y and dX equal the true-rank run, the gradients of the real entries equal the
    true-rank gradients and the gradients of the padding of A are exactly zero where B's padding rows are zero."""
    ranks, lens, scales = [8, 24, 64], [200, 77, 300], [2.0, 0.5, 1.0]
    k, n, rmax = 256, 320, 64
    w = wl.make_workload("true_rank", "bf16", k, n, ranks, lens, scales, seed=57, b_sigma=0.3)
    ref = DeviceLayer(w); ref.forward(); ref.backward(); ref.sync()
    dev = ref.device
    A_stack = torch.zeros((3, k, rmax), dtype=torch.bfloat16, device=dev)
    B_stack = torch.zeros((3, rmax, n), dtype=torch.bfloat16, device=dev)
    for i, r in enumerate(ranks):
        A_stack[i, :, :r] = ref.A[i]
        B_stack[i, :r, :] = ref.B[i]
    dA_stack, dB_stack = torch.full_like(A_stack, float("nan")), torch.full_like(B_stack, float("nan"))
    plan = ml.Plan(ml.BF16, w.T, k, n, [rmax] * 3, scales, w.offsets)
    Y, dX = torch.empty_like(ref.Y), torch.empty_like(ref.dX)
    S = torch.empty(w.T * rmax, dtype=torch.bfloat16, device=dev)
    ws = torch.zeros(max(plan.workspace_bytes(), 256), dtype=torch.uint8, device=dev)
    A, B = [A_stack[i] for i in range(3)], [B_stack[i] for i in range(3)]
    ml.multi_lora_fwd(plan, ref.X, ref.W, A, B, Y, S, ws)
    ml.multi_lora_bwd(plan, ref.dY, ref.X, ref.W, A, B, S, dX, [dA_stack[i] for i in range(3)], [dB_stack[i] for i in range(3)], ws)
    torch.cuda.synchronize()
    assert torch.equal(Y, ref.Y) and torch.equal(dX, ref.dX)            # zero padding adds exact zeros
    for i, r in enumerate(ranks):
        assert torch.equal(dA_stack[i, :, :r], ref.dA[i]) and torch.equal(dB_stack[i, :r, :], ref.dB[i])
        assert torch.all(dA_stack[i, :, r:] == 0)                        # dA = X^T (dY B^T): zero rows of B give zero columns
    # and against the oracle run on the stacked (padded) matrices themselves
    Ap = [np.pad(w.A[i], ((0, 0), (0, rmax - r))) for i, r in enumerate(ranks)]
    Bp = [np.pad(w.B[i], ((0, rmax - r), (0, 0))) for i, r in enumerate(ranks)]
    fw = orc.forward(w.X, w.W, Ap, Bp, scales, w.offsets)
    bw = orc.backward(w.dY, w.X, w.W, Ap, Bp, scales, w.offsets)
    assert rel_fro(to_host(Y), fw.Y) <= 1e-2 and row_rel_max(to_host(Y), fw.Y) <= 1e-2
    assert rel_fro(to_host(dX), bw.dX) <= 1e-2 and row_rel_max(to_host(dX), bw.dX) <= 1e-2
    for i in range(3):
        assert elem_excess(to_host(dA_stack[i]), bw.dA[i], "bf16") <= 1.0 and elem_excess(to_host(dB_stack[i]), bw.dB[i], "bf16") <= 1.0
        assert rel_fro(to_host(dB_stack[i]), bw.dB[i]) <= 1e-2           # the padding rows of dB are S_pad^T dY = 0 too
    plan.destroy()


@pytest.mark.parametrize("ranks,lens,k,n", [((128, 72, 96), (300, 64, 131), 256, 320), ((80,), (1,), 64, 64),
                                             ((128, 128), (700, 65), 1024, 192)])
def test_plans_with_only_wide_ranks(ranks, lens, k, n):
    """All ranks in 65..128 and multiples of 8, widths multiples of 64: the shrink kernels take the GEMM-tiled build
    (shared X / adapter tiles in a ring of direct global -> LDS loads); partial row blocks, ranks below 128."""
    w = wl.make_workload("wide_only", "bf16", k, n, list(ranks), list(lens), [0.5] * len(ranks), seed=58, b_sigma=0.3)
    check_full(w)


@pytest.mark.parametrize("ranks,lens,k,n", [((4, 12, 20, 36, 60, 8, 5), (300, 64, 131, 70, 129, 65, 40), 256, 320),
                                             ((4,), (1,), 64, 64),
                                             ((68, 100, 124, 4, 16), (130, 65, 200, 90, 64), 1024, 192)])
def test_ranks_that_are_multiples_of_4_but_not_of_8(ranks, lens, k, n):
    """Rows of such an A_i are 8-byte, not 16-byte, granular: the forward shrink keeps their adapter tile dense in LDS
    and the weight-gradient kernel loads their S / dS rows in 8-byte halves; mixed with ranks that take the other
    builds (multiples of 8, an odd rank) in one launch, narrow and wide."""
    w = wl.make_workload("rank_mod8_is_4", "bf16", k, n, list(ranks), list(lens), [0.5] * len(ranks), seed=59, b_sigma=0.3)
    check_full(w)


def test_single_token_segments():
    w = wl.make_workload("ones", "bf16", 256, 256, [4, 8, 16, 32, 5], [1, 1, 1, 1, 1],
                         [1.0, 2.0, 0.5, 0.25, 3.0], seed=53, b_sigma=0.3)
    check_full(w)


def test_error_does_not_grow_with_the_contraction_length():
    """fp32 accumulation and one rounding per output: the relative error of Y and dX is set by the bf16 rounding of the
    result (about 2^-9 / sqrt(3) = 1.1e-3, plus the rounded S / dS inside the LoRA term), whatever the contraction
    length; an accumulator narrower than fp32, or partial sums rounded on the way, would show as growth with k."""
    errs = {}
    for kk in (256, 1024, 4096, 16384):
        w = wl.make_workload(f"k{kk}", "bf16", kk, 256, [16, 64], [200, 120], [1.0, 0.25], seed=66, b_sigma=0.3)
        dl = DeviceLayer(w); dl.forward(); dl.backward(); dl.sync()
        fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
        errs[kk] = rel_fro(to_host(dl.Y), fw.Y)
        w2 = wl.make_workload(f"n{kk}", "bf16", 256, kk, [16, 64], [200, 120], [1.0, 0.25], seed=67, b_sigma=0.3)
        d2 = DeviceLayer(w2); d2.forward(); d2.backward(); d2.sync()
        bw = orc.backward(w2.dY, w2.X, w2.W, w2.A, w2.B, w2.scales, w2.offsets)
        errs[-kk] = rel_fro(to_host(d2.dX), bw.dX)
        dl.plan.destroy(); d2.plan.destroy()
    print("        relative error of Y by k and of dX by n:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert all(v <= 4e-3 for v in errs.values()), errs
    assert errs[16384] <= 1.5 * errs[256] and errs[-16384] <= 1.5 * errs[-256], errs


# ---- determinism and isolation ----------------------------------------------------------------------
def test_repeat_runs_are_bit_identical_and_adapters_are_isolated():
    w = wl.small_case(seed=61, dtype="bf16", k=512, n=512, ranks=(8, 64, 16), seg_lens=(300, 1200, 77),
                      scales=(2.0, 0.25, 1.0), b_sigma=0.3)
    dl = DeviceLayer(w); dl.forward(); dl.backward(); dl.sync()
    first = [t.clone() for t in (dl.Y, dl.dX, dl.S, *dl.dA, *dl.dB)]
    dl.forward(); dl.backward(); dl.sync()
    for a, b in zip(first, (dl.Y, dl.dX, dl.S, *dl.dA, *dl.dB)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # perturb adapter 1: rows of the other segments and the other adapters' gradients keep their bits
    dl.A[1].mul_(1.5); dl.B[1].add_(0.25)
    dl.forward(); dl.backward(); dl.sync()
    lo, hi = w.offsets[1], w.offsets[2]
    keep = torch.ones(w.T, dtype=torch.bool, device=dl.Y.device); keep[lo:hi] = False
    assert torch.equal(first[0][keep].view(torch.int16), dl.Y[keep].view(torch.int16))
    assert torch.equal(first[1][keep].view(torch.int16), dl.dX[keep].view(torch.int16))
    assert not torch.equal(first[0][lo:hi].view(torch.int16), dl.Y[lo:hi].view(torch.int16))
    for i in (0, 2):
        assert torch.equal(first[3 + i].view(torch.int16), dl.dA[i].view(torch.int16))
        assert torch.equal(first[6 + i].view(torch.int16), dl.dB[i].view(torch.int16))


def test_equal_length_batch_matches_same_data_run_as_ragged_neighbours():
    # equal token counts are just a special case of the ragged path (the paper's bmm fast path and
    # its grouped_mm path must agree): results for an adapter do not depend on its neighbours' lengths
    base = wl.small_case(seed=62, dtype="bf16", k=256, n=256, ranks=(16, 16, 16), seg_lens=(128, 128, 128),
                         scales=(1.0, 1.0, 1.0), b_sigma=0.3)
    dl, _, _ = check_full(base, label="equal lengths")          # the equal-length batch itself against the oracle
    # same middle adapter, neighbours shortened -> ragged offsets
    keep = np.r_[0:50, 128:256, 256:300]
    rag = wl.Workload(name="rag", dtype="bf16", T=len(keep), k=256, n=256, ranks=base.ranks, scales=base.scales,
                      offsets=[0, 50, 178, 222], X=base.X[keep], W=base.W, A=base.A, B=base.B, dY=base.dY[keep])
    dr, _, _ = check_full(rag, label="same adapter between ragged neighbours")
    assert rel_fro(to_host(dr.Y[50:178]), to_host(dl.Y[128:256])) <= 1e-6
    assert rel_fro(to_host(dr.dA[1]), to_host(dl.dA[1])) <= 1e-2
    assert rel_fro(to_host(dr.dX[50:178]), to_host(dl.dX[128:256])) <= 1e-6


# ---- error paths that need a live plan ----------------------------------------------------------------
def test_fwd_bwd_argument_errors():
    w = wl.small_case(seed=63, dtype="bf16", k=64, n=64, ranks=(8,), seg_lens=(10,), scales=(1.0,))
    dl = DeviceLayer(w)
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, dl.X, dl.W, dl.A, dl.B, dl.Y, dl.S, dl.workspace, 3, dl.stream)
    assert e.value.status == -9
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, dl.X, dl.W, dl.A, dl.B, dl.Y, dl.S, dl.workspace, 64, dl.stream)
    assert e.value.status == -9
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, None, dl.W, dl.A, dl.B, dl.Y, dl.S, dl.workspace, 0, dl.stream)
    assert e.value.status == -1
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, dl.X.data_ptr() + 2, dl.W, dl.A, dl.B, dl.Y, dl.S, dl.workspace, 0, dl.stream)
    assert e.value.status == -6
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, dl.X, dl.W, [None], dl.B, dl.Y, dl.S, dl.workspace, 0, dl.stream)
    assert e.value.status == -1
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_bwd(dl.plan, dl.dY, dl.X, dl.W, dl.A, dl.B, dl.S, dl.dX, dl.dA, dl.dB, None, 0, dl.stream)
    assert e.value.status == -7
    with pytest.raises(ml.MultiLoraError) as e:
        ml.multi_lora_fwd(dl.plan, dl.X, dl.W, [dl.A[0].data_ptr() + 8], dl.B, dl.Y, dl.S, dl.workspace, 0, dl.stream)
    assert e.value.status == -6
    dl.forward(); dl.backward(); dl.sync()      # the plan still works after rejected calls
