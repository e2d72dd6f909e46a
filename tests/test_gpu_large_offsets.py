"""Layers whose wide tensors (Y and dY, or X and dX) have more than 2^31 elements (4.65 GB in bf16): element and byte offsets
past the 32-bit range in every kernel that walks them (shrink / dShrink, fused GEMMs, weight gradients, expand-add).  Inputs are drawn on the GPU; the
oracle runs on the sampled rows, regrouped into a small workload with the same adapters: rows at the very start, around
2^31 elements, and the whole last adapter (300 tokens at the end of the buffer), whose S_i, dA_i and dB_i are compared
in full."""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import rel_fro

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,n", [(512, 14336), (14336, 512)])     # the wide side is Y / dY, then X / dX
def test_offsets_beyond_32_bits(k, n):
    ranks = [32, 16, 64, 8, 128, 16, 32, 64, 4, 16]
    lens = [18000] * 9 + [300]
    scales = [0.5, 1.0, 0.25, 2.0, 0.125, 1.0, 0.5, 0.25, 4.0, 1.0]
    dl = DeviceLayer.synthetic("large_offsets", "bf16", k, n, ranks, lens, scales, seed=77)
    T, off = dl.w.T, dl.w.offsets
    wide = max(k, n)
    assert T * wide > 2 ** 31 and T * wide * 2 > 2 ** 32
    print(f"[case] T={T} k={k} n={n}: the wide tensors have {T * wide} elements", flush=True)
    dl.Y.fill_(float("nan")); dl.dX.fill_(float("nan"))
    dl.forward(); dl.backward(); dl.sync()

    # sampled rows, grouped by adapter (so that the sample is itself a valid segmentation)
    wrap = (2 ** 31) // wide                   # the row in which the element index passes 2^31
    rows, sub_off = [], [0]
    for i in range(len(ranks)):
        lo, hi = off[i], off[i + 1]
        mine = {lo, hi - 1, (lo + hi) // 2}
        mine.update(r for r in (wrap - 1, wrap, wrap + 1) if lo <= r < hi)
        if i == len(ranks) - 1:
            mine = set(range(lo, hi))
        rows.extend(sorted(mine))
        sub_off.append(len(rows))
    idx = torch.tensor(rows, device=dl.device)
    f32 = lambda t: t.detach().to(torch.float32).cpu().numpy()       # exact widening of the bf16 inputs
    X, dY = f32(dl.X[idx]), f32(dl.dY[idx])
    W, A, B = f32(dl.W), [f32(a) for a in dl.A], [f32(b) for b in dl.B]
    fw = orc.forward(X, W, A, B, scales, sub_off)
    bw = orc.backward(dY, X, W, A, B, scales, sub_off)

    def check(tag, tol_y):
        errs = {"Y": rel_fro(to_host(dl.Y[idx]), fw.Y), "dX": rel_fro(to_host(dl.dX[idx]), bw.dX)}
        last = len(ranks) - 1
        errs["dA_last"] = rel_fro(to_host(dl.dA[last]), bw.dA[last])
        errs["dB_last"] = rel_fro(to_host(dl.dB[last]), bw.dB[last])
        errs["S_last"] = rel_fro(dl.S_list()[last], fw.S[last])
        # per-row check as well: one wrong row among hundreds would not move the Frobenius norm over the whole sample
        Yg, dXg = to_host(dl.Y[idx]), to_host(dl.dX[idx])
        errs["Y_row_max"] = max(rel_fro(Yg[j], fw.Y[j]) for j in range(len(rows)))
        errs["dX_row_max"] = max(rel_fro(dXg[j], bw.dX[j]) for j in range(len(rows)))
        print(f"        {tag}: " + ", ".join(f"{a} {b:.2e}" for a, b in errs.items()), flush=True)
        bad = {a: b for a, b in errs.items() if not b <= (tol_y if a.startswith(("Y", "dX")) else 1e-2)}
        assert not bad, (tag, bad)
        assert not torch.isnan(dl.Y).any() and not torch.isnan(dl.dX).any()

    check("fused", 1e-2)
    dl.Y.fill_(float("nan")); dl.dX.fill_(float("nan"))
    dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY)
    dl.backward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_LORA_ONLY)
    dl.sync()
    check("decoupled", 2e-2)
    dl.plan.destroy()
