"""The library's inter-task scheduler (host code behind the C ABI) against the oracle: the same canonical optimal schedule
(start times, GPUs, makespan) on random instances with integer durations - sums of integers are exact, so equality is
bit for bit -, validity and optimality (not identity) on real-valued ones, the paper's 8-GPU / 11-task shape within its
one-second budget, and identical decisions on random streams of arrivals, completions and polls."""
import time

import numpy as np
import pytest

from oracle import inter_task_oracle as its
from paper_2604_05426_amd import binding as ml


def test_hand_worked_cases():
    assert ml.schedule_tasks([3, 5, 2], [4, 4, 4], 4) == ([5.0, 0.0, 8.0], [[0, 1, 2, 3]] * 3, 10.0)
    assert ml.schedule_tasks([4, 3], [2, 1], 2, release=[0, 10]) == ([10.0, 0.0], [[0, 1], [0]], 14.0)
    assert ml.schedule_tasks([20, 5], [1, 1], 2, release=[0, 10]) == ([0.0, 10.0], [[0], [1]], 20.0)
    assert ml.schedule_tasks([], [], 3, now=7.5) == ([], [], 7.5)
    assert ml.schedule_tasks([10, 2, 2, 2, 2], [1] * 5, 2)[2] == 10.0       # shortest-first would need 14


@pytest.mark.parametrize("seed", range(8))
def test_same_canonical_schedule_as_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(25):
        n, G = int(rng.integers(0, 8)), int(rng.integers(1, 9))
        d = [int(x) for x in rng.integers(1, 12, size=n)]
        g = [int(x) for x in rng.choice([1, 1, 2, 4, G], size=n).clip(1, G)]
        now = float(rng.integers(0, 5))
        release = [now + float(x) for x in rng.choice([0, 0, 0, 3, 7], size=G)] if rng.random() < 0.5 else None
        starts, gpus, mk = ml.schedule_tasks(d, g, G, release, now)
        o_starts, o_mk = its.optimal_schedule(d, g, G, release, now)
        assert (starts, mk) == (o_starts, o_mk), (d, g, G, release, now)
        assert gpus == its.assign_gpus(o_starts, d, g, G, release, now)
        assert its.check_schedule(starts, gpus, d, g, G, release, now) == mk


def test_real_valued_durations_are_optimal_and_valid():
    rng = np.random.default_rng(9)
    for _ in range(40):
        n, G = int(rng.integers(1, 7)), int(rng.integers(1, 6))
        d = [float(x) for x in rng.uniform(0.5, 20.0, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        starts, gpus, mk = ml.schedule_tasks(d, g, G)
        assert its.check_schedule(starts, gpus, d, g, G) == pytest.approx(mk, rel=1e-12)
        assert mk == pytest.approx(its.optimal_schedule(d, g, G)[1], rel=1e-12)


def test_paper_sized_instance_within_a_second():
    # Sec. 8.3 (inter-task evaluation): 8 GPUs, 11 tasks of three sizes (4, 2 and 1 GPUs per task); durations synthetic
    rng = np.random.default_rng(11)
    for trial in range(5):
        g = [4, 4, 2, 2, 2, 1, 1, 1, 1, 1, 1]
        d = [float(x) for x in rng.integers(20, 400, size=11)]
        t0 = time.perf_counter()
        starts, gpus, mk = ml.schedule_tasks(d, g, 8)
        dt = time.perf_counter() - t0
        assert dt < 1.0, dt
        its.check_schedule(starts, gpus, d, g, 8)
        assert mk >= max(max(d), sum(di * gi for di, gi in zip(d, g)) / 8)
        # never worse than longest-first list scheduling
        lpt = its.list_schedule(sorted(range(11), key=lambda i: -d[i]), d, g, 8)[1]
        assert mk <= lpt


def test_search_budget_returns_a_valid_schedule():
    # 20 tasks: the exact search may run out of its budget; what comes back is valid, says whether it is proved optimal,
    # respects the lower bounds and is no worse than longest-first list scheduling
    rng = np.random.default_rng(12)
    g = [int(x) for x in rng.choice([1, 1, 1, 2, 2, 4], size=20)]
    d = [float(x) for x in rng.integers(20, 400, size=20)]
    t0 = time.perf_counter()
    starts, gpus, mk, proved = ml.schedule_tasks(d, g, 8, with_proof=True)
    assert time.perf_counter() - t0 < 20.0
    assert its.check_schedule(starts, gpus, d, g, 8) == pytest.approx(mk, rel=1e-12)
    assert mk >= max(max(d), sum(di * gi for di, gi in zip(d, g)) / 8)
    assert mk <= its.list_schedule(sorted(range(20), key=lambda i: (-g[i], -d[i])), d, g, 8)[1]
    assert ml.schedule_tasks([3, 5, 2], [4, 4, 4], 4, with_proof=True)[3] is True


@pytest.mark.parametrize("seed", range(8))
def test_event_loop_matches_oracle_on_random_streams(seed):
    rng = np.random.default_rng(200 + seed)
    G = int(rng.integers(1, 7))
    orc, lib = its.Cluster(G), ml.Cluster(G)
    now = 0.0
    for step in range(120):
        now += float(rng.integers(0, 4))
        u = rng.random()
        if u < 0.35 and len(orc.pending) < 6:
            d, g = float(rng.integers(1, 15)), int(rng.integers(1, G + 1))
            assert lib.submit(now, d, g) == orc.submit(now, d, g)
        elif u < 0.6 and orc.running:
            tid = list(orc.running)[int(rng.integers(len(orc.running)))]
            orc.complete(now, tid); lib.complete(now, tid)
        else:
            assert lib.poll(now) == orc.poll(now)
        plan, mk = lib.plan()
        assert plan == orc.plan and mk == orc.planned_makespan
    lib.destroy()


def test_argument_errors():
    with pytest.raises(ml.MultiLoraError):
        ml.schedule_tasks([1.0], [3], 2)             # needs more GPUs than the cluster has
    with pytest.raises(ml.MultiLoraError):
        ml.schedule_tasks([0.0], [1], 2)
    with pytest.raises(ml.MultiLoraError):
        ml.schedule_tasks([1.0] * 25, [1] * 25, 2)
    with pytest.raises(ml.MultiLoraError):
        ml.Cluster(0)
    c = ml.Cluster(2)
    with pytest.raises(ml.MultiLoraError):
        c.complete(0.0, 5)
    with pytest.raises(ml.MultiLoraError):
        c.submit(0.0, 1.0, 3)
    c.destroy()
