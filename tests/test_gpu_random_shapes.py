"""Seeded random layers against the oracle: widths that are and are not multiples of 8 (MFMA and FMA kernels) and of 64, ranks
from 0 to 128 including odd ones and the class boundaries, segment lengths around the 64-row block and 256-row tile
boundaries including empty ones, in the fused mode, the decoupled mode (frozen-weight pass, then LoRA-only pass in
place) and with gradient accumulation."""
import numpy as np
import pytest

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import rel_fro

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(6))
def test_random_layers(block):
    for case in range(block * 12, block * 12 + 12):
        rng = np.random.default_rng(9000 + case)
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        if block >= 4:      # widths that are multiples of 64: the shrink kernels take their tiled form
            k, n = int(rng.integers(1, 30)) * 64, int(rng.integers(1, 30)) * 64
        else:
            k = int(rng.integers(1, 200)) * 8 if rng.random() < 0.85 else int(rng.integers(1, 300))
            n = int(rng.integers(1, 200)) * 8 if rng.random() < 0.85 else int(rng.integers(1, 300))
        N = int(rng.integers(1, 7))
        ranks = [int(rng.choice([0, 1, 3, 4, 8, 16, 24, 32, 40, 64, 65, 96, 100, 128])) for _ in range(N)]
        lens = [int(rng.choice([0, 1, 2, 63, 64, 65, 127, 255, 256, 257, 300, 700, 1500])) for _ in range(N)]
        scales = [float(rng.choice([0.125, 0.5, 1.0, 2.0, 3.0])) for _ in range(N)]
        mode = int(rng.integers(0, 3))
        print(f"[case {case}] {dtype} k={k} n={n} ranks={ranks} lens={lens} mode={mode}", flush=True)
        w = wl.make_workload(f"random{case}", dtype, k, n, ranks, lens, scales, seed=9000 + case, b_sigma=0.3)
        tol = 1e-2 if dtype == "bf16" else 1e-5
        fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
        bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
        dl = DeviceLayer(w)
        if mode == 0:
            dl.forward(); dl.backward()
        elif mode == 1:
            dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY)
            dl.backward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_LORA_ONLY)
        else:
            dl.forward()
            for t in dl.dA + dl.dB:
                t.zero_()
            dl.backward(ml.FLAG_ACCUM_GRADS)
        dl.sync()
        two = 2.0 if mode == 1 else 1.0      # the decoupled mode stores the frozen-weight result before adding: two roundings
        if w.T:
            assert rel_fro(to_host(dl.Y), fw.Y) <= two * tol and rel_fro(to_host(dl.dX), bw.dX) <= two * tol, case
        for i in range(w.N):
            assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= tol and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= tol, (case, i)
        dl.plan.destroy()
