"""GPU parity at the full sizes of the five benchmark configs, in the launch configuration the
benchmark times.  Config 1 (tiny) is compared in full in test_gpu_parity.py; configs 2-5 are
compared on sampled outputs the oracle computes one by one: Y and dX on rows at segment ends,
around tile boundaries and at random positions, S and dS in full for a few adapters, and dA_i,
dB_i on sampled rows / columns (each sampled element is still the full token reduction)."""
import time

import numpy as np
import pytest

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import elem_excess, rel_fro, row_rel_max, sample_cols

pytestmark = pytest.mark.gpu


def pick_adapters(w):
    cand = [0, w.N - 1, int(np.argmax(w.ranks)), int(np.argmin(w.seg_lens)), int(np.argmax(w.seg_lens))]
    out = []
    for c in cand:
        if c not in out and w.seg_lens[c] > 0:
            out.append(c)
    return out[:4]


def pick_rows(w, adapters, tile_rows, seed):
    rng = np.random.default_rng(seed)
    rows = set()
    for i in adapters:
        lo, hi = w.offsets[i], w.offsets[i + 1]
        rows.update([lo, hi - 1, int(rng.integers(lo, hi)), int(rng.integers(lo, hi))])
        b = ((lo // tile_rows) + 1) * tile_rows          # first tile boundary inside the segment
        if b < hi:
            rows.update([b - 1, b])
        b2 = ((hi - 1) // tile_rows) * tile_rows         # last tile boundary inside the segment
        if lo < b2 < hi:
            rows.update([b2 - 1, b2])
    return np.array(sorted(r for r in rows if 0 <= r < w.T), dtype=np.int64)


@pytest.mark.parametrize("index", [1, 2, 3, 4])
def test_config_full_size_sampled(index):
    t0 = time.time()
    print(f"[case] config {index + 1} ({wl.CONFIG_NAMES[index]}): drawing inputs", flush=True)
    w = wl.config(index)
    print(f"        T={w.T} k={w.k} n={w.n} N={w.N} ranks={w.ranks} lens={w.seg_lens} ({time.time() - t0:.1f}s)", flush=True)
    dl = DeviceLayer(w)
    dl.forward(); dl.backward(); dl.sync()
    print(f"        GPU done ({time.time() - t0:.1f}s)", flush=True)
    geo = dl.plan.geometry()
    assert geo[ml.GEO_USES_MFMA] == 1
    ads = pick_adapters(w)
    rows = pick_rows(w, ads, geo[ml.GEO_GEMM_TILE_ROWS], seed=index)
    ycols = sample_cols(w.n, geo[ml.GEO_GEMM_TILE_COLS], 320, seed=index)
    xcols = sample_cols(w.k, geo[ml.GEO_GEMM_TILE_COLS], 320, seed=index + 7)
    fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets, rows=rows, cols=ycols, adapters=ads)
    print(f"        oracle forward done ({time.time() - t0:.1f}s)", flush=True)
    bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets, S=fw.S, rows=rows, cols=xcols,
                      a_rows=xcols, b_cols=ycols, adapters=ads)
    print(f"        oracle backward done ({time.time() - t0:.1f}s)", flush=True)
    errs = {}
    Yg = to_host(dl.Y[rows.tolist()])[:, ycols]
    dXg = to_host(dl.dX[rows.tolist()])[:, xcols]
    errs["Y"], errs["dX"] = rel_fro(Yg, fw.Y), rel_fro(dXg, bw.dX)
    errs["Y_row_max"], errs["dX_row_max"] = row_rel_max(Yg, fw.Y), row_rel_max(dXg, bw.dX)     # every sampled row by itself
    S, dS = dl.S_list(), dl.dS_list()
    elem = {}
    for i in ads:
        got = {"S": S[i], "dS": dS[i], "dA": to_host(dl.dA[i])[xcols], "dB": to_host(dl.dB[i])[:, ycols]}
        want = {"S": fw.S[i], "dS": bw.dS[i], "dA": bw.dA[i], "dB": bw.dB[i]}
        for name in got:
            errs[f"{name}{i}"] = rel_fro(got[name], want[name])
            elem[f"{name}{i}"] = elem_excess(got[name], want[name], "bf16")                       # and every element by itself
    worst = max(errs.items(), key=lambda kv: kv[1])
    worst_e = max(elem.items(), key=lambda kv: kv[1])
    print(f"        worst {worst[0]} = {worst[1]:.3e}; worst element {worst_e[0]} at {worst_e[1]:.2f} of its bound  ({time.time() - t0:.1f}s)", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= 1e-2}
    bad.update({k + "_elem": v for k, v in elem.items() if not v <= 1.0})
    assert not bad, bad
    # properties that hold at any size: every output element was written (outputs start as NaN)
    import torch
    assert not torch.isnan(dl.Y).any() and not torch.isnan(dl.dX).any() and not torch.isnan(dl.S[: w.R1]).any()
    for i in range(w.N):
        assert not torch.isnan(dl.dA[i]).any() and not torch.isnan(dl.dB[i]).any()
    # the decoupled form at the same size (frozen-weight pass, then the LoRA-only pass in place: the expand-add kernels,
    # which choose their cache hints by the size of the output); Y / dX are rounded twice there
    dl.Y.fill_(float("nan")); dl.dX.fill_(float("nan"))
    dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY)
    dl.backward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_LORA_ONLY)
    dl.sync()
    Y2, dX2 = to_host(dl.Y[rows.tolist()])[:, ycols], to_host(dl.dX[rows.tolist()])[:, xcols]
    e2 = {"Y": rel_fro(Y2, fw.Y), "dX": rel_fro(dX2, bw.dX), "Y_row_max": row_rel_max(Y2, fw.Y), "dX_row_max": row_rel_max(dX2, bw.dX)}
    for i in ads:
        e2[f"dA{i}"] = rel_fro(to_host(dl.dA[i])[xcols], bw.dA[i])
        e2[f"dB{i}"] = rel_fro(to_host(dl.dB[i])[:, ycols], bw.dB[i])
    print(f"        decoupled form: worst {max(e2.values()):.3e}  ({time.time() - t0:.1f}s)", flush=True)
    bad = {k: v for k, v in e2.items() if not v <= (2e-2 if k.startswith(("Y", "dX")) else 1e-2)}
    assert not bad, bad
    assert not torch.isnan(dl.Y).any() and not torch.isnan(dl.dX).any()


@pytest.mark.parametrize("index", [2, 4])
def test_config_full_size_repeat_runs_are_bit_identical(index):
    """A property that holds at any size and needs no oracle: every reduction has a fixed order (no atomics), so two
    steps on the same inputs give the same bits - at full size, where the weight gradients of config 3 go through
    chunk partials and the fixed-order sum, and config 5 runs tens of thousands of work groups.  Any data race shows here."""
    import torch
    dtype, k, n, ranks, lens, scales, seed, _ = wl.config_shape(index)
    print(f"[case] config {index + 1}: repeat-run determinism at full size", flush=True)
    dl = DeviceLayer.synthetic(f"config{index + 1}", dtype, k, n, ranks, lens, scales, seed)
    outs = lambda: [dl.Y, dl.dX, dl.S] + dl.dA + dl.dB
    dl.forward(); dl.backward(); dl.sync()
    first = [t.clone() for t in outs()]
    for t in outs():
        t.fill_(float("nan"))
    dl.forward(); dl.backward(); dl.sync()
    for a, b in zip(first, outs()):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert not any(bool(torch.isnan(t).any()) for t in outs())
    dl.plan.destroy()
