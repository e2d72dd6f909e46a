"""Pins of the inter-task scheduling oracle (Sec. 6.2): closed forms, brute force straight on the definition, the
paper's constraints as a checker, classic special cases."""
import itertools

import numpy as np
import pytest

from oracle import inter_task_oracle as its


def test_closed_forms():
    # every task needs the whole cluster: they run one after the other
    starts, mk = its.optimal_schedule([3, 5, 2], [4, 4, 4], 4)
    assert mk == 10 and starts == [5, 0, 8]       # candidate order: longest first among equal GPU counts
    # as many single-GPU tasks as GPUs: all at once
    starts, mk = its.optimal_schedule([3, 5, 2, 4], [1, 1, 1, 1], 4)
    assert mk == 5 and starts == [0, 0, 0, 0]
    # unit tasks on G GPUs: ceil(n / G) rounds
    for n, G in [(7, 3), (6, 3), (1, 5), (8, 2)]:
        _, mk = its.optimal_schedule([1] * n, [1] * n, G)
        assert mk == -(-n // G)
    # nothing to do
    assert its.optimal_schedule([], [], 3) == ([], 0.0)
    assert its.optimal_schedule([], [], 3, now=7.5) == ([], 7.5)


def test_motivating_case_short_first_wastes_gpus():
    # Sec. 3 (motivation): placing the short tasks first leaves GPUs idle while the long task runs alone
    d, g, G = [10, 2, 2, 2, 2], [1, 1, 1, 1, 1], 2
    sjf = sorted(range(5), key=lambda i: d[i])
    _, mk_sjf = its.list_schedule(sjf, d, g, G)
    _, mk_opt = its.optimal_schedule(d, g, G)
    assert mk_sjf == 14 and mk_opt == 10


def test_lower_bounds_hold_and_schedule_satisfies_the_papers_constraints():
    rng = np.random.default_rng(5)
    for _ in range(60):
        n, G = int(rng.integers(1, 7)), int(rng.integers(1, 6))
        d = [int(x) for x in rng.integers(1, 9, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        starts, mk = its.optimal_schedule(d, g, G)
        gpus = its.assign_gpus(starts, d, g, G)
        assert its.check_schedule(starts, gpus, d, g, G) == mk
        assert mk >= max(d) and mk * G >= sum(di * gi for di, gi in zip(d, g))


def test_against_brute_force_on_the_definition():
    # integer data: an optimal schedule with integer starts exists; enumerate all start vectors
    rng = np.random.default_rng(6)
    for _ in range(40):
        n, G = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        d = [int(x) for x in rng.integers(1, 5, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        _, mk = its.optimal_schedule(d, g, G)
        assert mk == its.time_indexed_optimum(d, g, G, horizon=sum(d))


def test_single_gpu_tasks_reduce_to_machine_assignment():
    # all g_i = 1: P || C_max; brute force over assignments of tasks to machines (a different formulation)
    rng = np.random.default_rng(7)
    for _ in range(30):
        n, G = int(rng.integers(1, 7)), int(rng.integers(1, 4))
        d = [int(x) for x in rng.integers(1, 10, size=n)]
        best = min(max(sum(d[i] for i in range(n) if a[i] == m) for m in range(G))
                   for a in itertools.product(range(G), repeat=n))
        _, mk = its.optimal_schedule(d, [1] * n, G)
        assert mk == best


def test_release_times_and_now():
    # GPU 1 is held until t = 10; a 2-GPU task has to wait for it, a 1-GPU task runs at once on GPU 0
    starts, mk = its.optimal_schedule([4, 3], [2, 1], 2, release=[0, 10], now=0)
    assert starts == [10, 0] and mk == 14
    gpus = its.assign_gpus(starts, [4, 3], [2, 1], 2, release=[0, 10])
    assert gpus == [[0, 1], [0]]
    its.check_schedule(starts, gpus, [4, 3], [2, 1], 2, release=[0, 10])
    # a long 1-GPU task placed first must not block the GPU that is released later
    starts, mk = its.optimal_schedule([20, 5], [1, 1], 2, release=[0, 10], now=0)
    assert mk == 20 and starts == [0, 10]
    # nothing starts before `now`
    starts, mk = its.optimal_schedule([2, 2], [1, 1], 1, now=3.0)
    assert sorted(starts) == [3.0, 5.0] and mk == 7.0


def test_checker_rejects_planted_mistakes():
    d, g, G = [4, 3], [2, 1], 2
    with pytest.raises(AssertionError):
        its.check_schedule([0, 0], [[0, 1], [0]], d, g, G)              # overlap on GPU 0
    with pytest.raises(AssertionError):
        its.check_schedule([0, 4], [[0], [0]], d, g, G)                 # task 0 holds one GPU instead of two
    with pytest.raises(AssertionError):
        its.check_schedule([0, 4], [[0, 1], [1]], d, g, G, release=[0, 6])   # GPU 1 not yet released
    assert its.check_schedule([0, 4], [[0, 1], [1]], d, g, G) == 7


def test_canonical_choice_among_optimal_schedules():
    # two equal tasks: the lower index goes first; candidate order is (g desc, d desc, index)
    starts, mk = its.optimal_schedule([5, 5], [1, 1], 1)
    assert starts == [0, 5]
    assert its.candidate_order([3, 9, 9, 1], [1, 2, 2, 4]) == [3, 1, 2, 0]


def test_cluster_event_loop():
    c = its.Cluster(2)
    a = c.submit(0.0, 10.0, 1)
    b = c.submit(0.0, 4.0, 2)
    # optimum: 2-GPU task first (0..4), then the long one (4..14); or long first and the pair waits (10..14): both 14;
    # candidate order puts the 2-GPU task first
    assert c.planned_makespan == 14.0
    assert c.poll(0.0) == [(b, [0, 1])]
    assert c.poll(1.0) == []
    # the pair finishes early (its adapters exited): the freed GPUs are backfilled at once
    c.complete(2.5, b)
    assert c.poll(2.5) == [(a, [0])]
    assert c.planned_makespan == 12.5
    e = c.submit(3.0, 1.0, 1)
    assert c.poll(3.0) == [(e, [1])]
    f = c.submit(3.5, 2.0, 2)       # needs both GPUs: after the long task's estimated end
    assert c.plan[f] == 12.5 and c.poll(3.5) == []
    c.complete(4.0, e)
    # the long task overruns its estimate: nothing can start, the plan moves with the clock
    assert c.poll(13.0) == [] and c.plan[f] == 13.0
    c.complete(13.5, a)
    assert c.poll(13.5) == [(f, [0, 1])]
    with pytest.raises(KeyError):
        c.complete(14.0, a)
