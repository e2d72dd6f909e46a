"""GPU tests of properties around the layer's arithmetic: co-located jobs stay isolated when one of them has diverged
to Inf / NaN weights (paper Sec. 4.1, Pattern 1: divergence is expected, and it must not reach the neighbours), plans
made from plans made from plans outlive their ancestors, and the number of launches per step does not depend on the
number of adapters (Sec. 5.1: O(1) launches)."""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import rel_fro, row_rel_max

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.contiguous().view(torch.int16)


@pytest.mark.parametrize("poison", ["B_inf", "A_nan", "B_inf_second_rank_pass"])
@pytest.mark.parametrize("decoupled", [False, True])
def test_non_finite_weights_of_one_adapter_do_not_reach_its_neighbours(poison, decoupled):
    # segments 300 / 1200 / 77 rows: the 256-row tiles of the fused GEMM straddle both boundaries of adapter 1
    w = wl.small_case(seed=65, dtype="bf16", k=512, n=512, ranks=(8, 128, 16), seg_lens=(300, 1200, 77),
                      scales=(2.0, 0.25, 1.0), b_sigma=0.3)
    print(f"[case] isolation poison={poison} decoupled={decoupled}", flush=True)
    dl = DeviceLayer(w)

    def step():
        if decoupled:
            dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY)
            dl.backward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_LORA_ONLY)
        else:
            dl.forward(); dl.backward()
        dl.sync()

    step()
    clean = [t.clone() for t in (dl.Y, dl.dX, *dl.dA, *dl.dB)]
    assert all(bool(torch.isfinite(t).all()) for t in clean)
    if poison == "B_inf":
        dl.B[1][3, 17] = float("inf"); ycol, xcol = 17, None
    elif poison == "B_inf_second_rank_pass":
        dl.B[1][100, 300] = float("-inf"); ycol, xcol = 300, None
    else:
        dl.A[1][5, 2] = float("nan"); ycol, xcol = None, 5
    step()
    lo, hi = w.offsets[1], w.offsets[2]
    keep = torch.ones(w.T, dtype=torch.bool, device=dl.Y.device)
    keep[lo:hi] = False
    # the neighbours keep their bits: rows of the other segments, gradients of the other adapters
    assert torch.equal(_bits(clean[0][keep]), _bits(dl.Y[keep]))
    assert torch.equal(_bits(clean[1][keep]), _bits(dl.dX[keep]))
    for i in (0, 2):
        assert torch.equal(_bits(clean[2 + i]), _bits(dl.dA[i])) and torch.equal(_bits(clean[5 + i]), _bits(dl.dB[i]))
    # the diverged adapter sees what the plain definition gives it: non-finite where its Inf / NaN enters, its old bits elsewhere
    if ycol is not None:       # B_1[rho, ycol] = Inf: column ycol of its Y rows; every column of its dX rows (through dS)
        assert not bool(torch.isfinite(dl.Y[lo:hi, ycol]).any())
        others = [c for c in range(w.n) if c != ycol]
        assert torch.equal(_bits(clean[0][lo:hi][:, others]), _bits(dl.Y[lo:hi][:, others]))
        assert not bool(torch.isfinite(dl.dX[lo:hi]).any())
    else:                      # A_1[xcol, rho] = NaN: every column of its Y rows (through S); column xcol of its dX rows
        assert not bool(torch.isfinite(dl.Y[lo:hi]).any())
        assert not bool(torch.isfinite(dl.dX[lo:hi, xcol]).any())
        others = [c for c in range(w.k) if c != xcol]
        assert torch.equal(_bits(clean[1][lo:hi][:, others]), _bits(dl.dX[lo:hi][:, others]))
    dl.plan.destroy()


def test_plans_made_from_plans_outlive_their_ancestors():
    ranks, lens, scales = [8, 0, 100, 16], [150, 64, 300, 77], [2.0, 1.0, 0.4, 0.125]
    wa = wl.make_workload("a", "bf16", 256, 320, ranks, lens, scales, seed=73, b_sigma=0.3)
    wc = wl.make_workload("c", "bf16", 192, 512, ranks, lens, scales, seed=74, b_sigma=0.3)
    a = ml.Plan(ml.BF16, wa.T, wa.k, wa.n, ranks, scales, wa.offsets)
    b = ml.Plan.like(a, 128, 64)
    c = ml.Plan.like(b, wc.k, wc.n)             # C like B like A: C's tables live in A's allocation
    own = ml.Plan(ml.BF16, wc.T, wc.k, wc.n, ranks, scales, wc.offsets)
    want = {t: own.dump(t) for t in range(5)}
    assert c.geometry() == own.geometry() and c.workspace_bytes() == own.workspace_bytes()
    a.destroy(); b.destroy(); own.destroy()
    torch.cuda.synchronize()
    junk = [torch.full((1 << 18,), -1, dtype=torch.int32, device="cuda:0") for _ in range(8)]   # reuse freed memory, if any was freed
    torch.cuda.synchronize()
    for t in range(5):
        assert c.dump(t) == want[t], t
    dl = DeviceLayer(wc)
    dl.plan.destroy()
    dl.plan = c
    dl.forward(); dl.backward(); dl.sync()
    fw = orc.forward(wc.X, wc.W, wc.A, wc.B, wc.scales, wc.offsets)
    bw = orc.backward(wc.dY, wc.X, wc.W, wc.A, wc.B, wc.scales, wc.offsets)
    assert rel_fro(to_host(dl.Y), fw.Y) <= 1e-2 and row_rel_max(to_host(dl.Y), fw.Y) <= 1e-2
    assert rel_fro(to_host(dl.dX), bw.dX) <= 1e-2
    for i in range(wc.N):
        assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= 1e-2 and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= 1e-2
    del junk
    c.destroy()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_launches_per_step_do_not_depend_on_the_number_of_adapters(dtype):
    """Same rank classes and the same token chunking (one chunk per adapter), 1 / 8 / 32 / 100 adapters: a step records
    the same kernels in the same order.  (The first step of a plan uploads the per-adapter pointers in batches of 32
    adapters; later steps with the same buffers skip that, which is the steady state counted here.)"""
    seen = {}
    for N in (1, 8, 32, 100):
        ranks = [[16, 96][i % 2] for i in range(N)] if N > 1 else [16]
        if N == 1:
            ranks = [96]      # the wide class alone takes the same builds as a mixed plan
        w = wl.make_workload(f"n{N}", dtype, 128, 192, ranks, [40] * N, [1.0] * N, seed=80 + N, b_sigma=0.3)
        dl = DeviceLayer(w)
        dl.forward(); dl.backward(); dl.sync()
        dl.plan.profile_begin(64)
        dl.forward(); dl.backward()
        recs = dl.plan.profile_end(64)
        dl.sync()
        seen[N] = [kid for kid, _ in recs]
        print(f"[case] {dtype} N={N}: {len(recs)} launches per step: {[ml.KERNEL_NAMES[k] for k in seen[N]]}", flush=True)
        dl.plan.destroy()
    assert seen[8] == seen[32] == seen[100]
    assert len(seen[1]) <= len(seen[8])          # a single rank class launches one weight-gradient kernel fewer


def test_adapter_permutation_moves_rows_and_leaves_every_bit_alone():
    """Permuting the adapters (segments, ranks, scales, matrices together) permutes the rows of Y and dX and leaves every
    dA_i, dB_i unchanged - bit for bit: a row's result does not depend on where in the flat buffer, in which tile or next
    to which neighbours it sits.  (The oracle has the same property exactly; here it is the kernels' tiling that is on trial:
    segments that are not multiples of any tile, three rank classes.)"""
    ranks, lens, scales = [8, 100, 0, 33, 64], [300, 210, 70, 129, 515], [2.0, 0.25, 1.0, 0.5, 0.125]
    w = wl.make_workload("perm_base", "bf16", 320, 264, ranks, lens, scales, seed=75, b_sigma=0.3)
    perm = [3, 0, 4, 2, 1]
    rows = np.concatenate([np.arange(w.offsets[i], w.offsets[i + 1]) for i in perm])
    off = [0]
    for i in perm:
        off.append(off[-1] + lens[i])
    wp = wl.Workload(name="perm", dtype="bf16", T=w.T, k=w.k, n=w.n, ranks=[ranks[i] for i in perm], scales=[scales[i] for i in perm],
                     offsets=off, X=w.X[rows], W=w.W, A=[w.A[i] for i in perm], B=[w.B[i] for i in perm], dY=w.dY[rows])
    a, b = DeviceLayer(w), DeviceLayer(wp)
    for d in (a, b):
        d.forward(); d.backward(); d.sync()
    idx = torch.tensor(rows, device=a.Y.device)
    assert torch.equal(_bits(a.Y[idx]), _bits(b.Y)) and torch.equal(_bits(a.dX[idx]), _bits(b.dX))
    for j, i in enumerate(perm):
        assert torch.equal(_bits(a.dA[i]), _bits(b.dA[j])) and torch.equal(_bits(a.dB[i]), _bits(b.dB[j])), (i, j)
    a.plan.destroy(); b.plan.destroy()


@pytest.mark.parametrize("k,n,total", [(384, 1544, 10540), (1024, 520, 8192 + 77)])
def test_grouped_row_bands_change_the_tile_order_and_no_bit(k, n, total):
    """MLORA_FLAG_GROUP_BANDS (what the library does by itself for weights larger than half the Infinity Cache) interleaves
    four 2048-row bands by groups of four column tiles.  The shapes put every branch of that numbering on trial: five full
    bands and a short one (one group of four and a single band behind it), column counts that are not multiples of four tiles
    (one whole group plus three tiles, one of them ragged; fewer than four tiles: no whole group at all), exactly four bands
    and a 77-row one.  Every tile must be computed exactly once: same bits as the ungrouped order, which the parity tests
    hold against the oracle, and the sampled rows are held against the oracle here as well."""
    lens = [1500, 2300, 700, total - 1500 - 2300 - 700 - 1300, 1300]
    ranks, scales = [16, 128, 0, 40, 64], [2.0, 0.25, 1.0, 0.5, 1.0]
    w = wl.make_workload("bands", "bf16", k, n, ranks, lens, scales, seed=91, b_sigma=0.3)
    print(f"[case] grouped bands k={k} n={n} T={w.T}", flush=True)
    dl = DeviceLayer(w)
    dl.forward(); dl.backward(); dl.sync()
    plain = [t.clone() for t in (dl.Y, dl.dX, *dl.dA, *dl.dB)]
    dl.Y.fill_(-3.0); dl.dX.fill_(-3.0)
    dl.forward(ml.FLAG_GROUP_BANDS); dl.backward(ml.FLAG_GROUP_BANDS); dl.sync()
    for a, b in zip(plain, (dl.Y, dl.dX, *dl.dA, *dl.dB)):
        assert torch.equal(_bits(a), _bits(b))
    rows = np.unique(np.concatenate([np.arange(0, w.T, 251), np.arange(w.T - 40, w.T), [2047, 2048, 8191, 8192]]))
    rows = rows[rows < w.T]
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets, rows=rows)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets, S=fw.S, rows=rows)
    assert rel_fro(to_host(dl.Y[rows.tolist()]), fw.Y) < 1e-2 and row_rel_max(to_host(dl.Y[rows.tolist()]), fw.Y) <= 1e-2
    assert rel_fro(to_host(dl.dX[rows.tolist()]), bw.dX) < 1e-2 and row_rel_max(to_host(dl.dX[rows.tolist()]), bw.dX) <= 1e-2
    dl.plan.destroy()


def test_grouped_row_bands_flag_is_accepted_and_ignored_by_the_fp32_path():
    w = wl.small_case(seed=93, dtype="f32", k=96, n=72, ranks=(4, 16), seg_lens=(150, 300), scales=(2.0, 0.5), b_sigma=0.3)
    dl = DeviceLayer(w)
    dl.forward(); dl.backward(); dl.sync()
    plain = [t.clone() for t in (dl.Y, dl.dX, *dl.dA, *dl.dB)]
    dl.forward(ml.FLAG_GROUP_BANDS); dl.backward(ml.FLAG_GROUP_BANDS); dl.sync()
    for a, b in zip(plain, (dl.Y, dl.dX, *dl.dA, *dl.dB)):
        assert torch.equal(a.contiguous().view(torch.int32), b.contiguous().view(torch.int32))
    dl.plan.destroy()
