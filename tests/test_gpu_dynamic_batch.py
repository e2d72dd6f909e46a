"""The loop the paper describes around the layer (Sec. 4 and Sec. 6.1): the monitor makes jobs exit, the scheduler
backfills, the running set becomes the next step's segmentation, and the layer is re-planned and stepped.  Every round's
GPU result is checked against the oracle for that round's segmentation."""
import numpy as np
import pytest
import torch

from oracle import multilora_oracle as orc
from paper_2604_05426_amd import binding as ml
from paper_2604_05426_amd import workloads as wl
from paper_2604_05426_amd.harness import DeviceLayer, to_host
from util import rel_fro

pytestmark = pytest.mark.gpu


def test_exit_backfill_replan_step():
    L, k, n = 64, 256, 320
    jobs = {j: {"batch": [4, 4, 2, 2, 1, 1, 4, 2][j], "rank": [8, 16, 32, 64, 128, 4, 16, 8][j]} for j in range(8)}
    sched = ml.Admission(0.0, 1.0 / L, 9.0, 1.0, L)               # Mhat(B) = B: at most 9 samples per step
    mon = ml.Monitor(len(jobs), 1.0, 2, 1e-3, 0.1, 1, 1)
    for j, d in jobs.items():
        sched.submit(j, d["batch"])
    sched.fill()
    seen = []
    for rnd in range(4):
        running = sched.running()
        seen.append([j for j, _ in running])
        ranks = [jobs[j]["rank"] for j, _ in running]
        lens = [b * L for _, b in running]
        w = wl.make_workload(f"round{rnd}", "bf16", k, n, ranks, lens, [2.0] * len(ranks), seed=300 + rnd, b_sigma=0.3)
        dl = DeviceLayer(w)
        dl.forward(); dl.backward(); dl.sync()
        fw = orc.forward(w.X, w.W, w.A, w.B, w.scales, w.offsets)
        bw = orc.backward(w.dY, w.X, w.W, w.A, w.B, w.scales, w.offsets)
        assert rel_fro(to_host(dl.Y), fw.Y) <= 1e-2 and rel_fro(to_host(dl.dX), bw.dX) <= 1e-2
        for i in range(w.N):
            assert rel_fro(to_host(dl.dA[i]), bw.dA[i]) <= 1e-2 and rel_fro(to_host(dl.dB[i]), bw.dB[i]) <= 1e-2
        dl.plan.destroy()
        # synthetic losses: the first running job overfits (validation 50 % above training), the others are fine
        for pos, (j, _) in enumerate(running):
            mon.train_loss(j, 1.0)
            decision = mon.val_loss(j, 1.5 if pos == 0 else 1.02)
            if decision != ml.EXIT_CONTINUE:
                assert decision == ml.EXIT_OVERFITTING and pos == 0
                sched.exit(j)
    # every round lost its first job and was refilled from the queue while something was pending
    assert seen[0] == [0, 1, 4] and seen[1][0] == 1 and 0 not in seen[1]
    assert all(sum(jobs[j]["batch"] for j in s) <= 9 for s in seen)
    assert len({tuple(s) for s in seen}) == 4
