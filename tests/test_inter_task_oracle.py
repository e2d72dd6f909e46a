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


# ---- the paper's program as printed, and the canonical choice pinned without the oracle's own enumeration ----------

def _subsets(G, size):
    return [list(c) for c in itertools.combinations(range(G), size)]


def test_big_m_program_agrees_with_the_plain_checker():
    rng = np.random.default_rng(8)
    seen_bad = 0
    for _ in range(80):
        n, G = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        d = [int(x) for x in rng.integers(1, 6, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        starts, mk = its.optimal_schedule(d, g, G)
        gpus = its.assign_gpus(starts, d, g, G)
        assert its.check_big_m(starts, gpus, d, g, G, mk)
        assert not its.check_big_m(starts, gpus, d, g, G, mk - 0.5)          # C_max below a completion time
        # a random schedule (random starts, random GPU sets): both statements of the constraints agree on it
        # (all tasks end by M = sum d, the range in which M is big enough to switch a constraint off)
        rs = [int(rng.integers(0, sum(d) - d[i] + 1)) for i in range(n)]
        rg = [[int(q) for q in rng.choice(G, size=g[i], replace=False)] for i in range(n)]
        try:
            its.check_schedule(rs, rg, d, g, G)
            plain_ok = True
        except AssertionError:
            plain_ok = False
            seen_bad += 1
        assert its.check_big_m(rs, rg, d, g, G, max(s + di for s, di in zip(rs, d))) == plain_ok
    assert seen_bad > 10


def test_optimum_of_the_big_m_program_by_brute_force():
    # tiny integer instances: every start vector x every GPU assignment through the program as printed
    rng = np.random.default_rng(9)
    for _ in range(25):
        n, G = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        d = [int(x) for x in rng.integers(1, 4, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        best = None
        for starts in itertools.product(range(sum(d)), repeat=n):
            mk = max(s + di for s, di in zip(starts, d))
            if best is not None and mk >= best:
                continue
            for sets in itertools.product(*[_subsets(G, gi) for gi in g]):
                if its.check_big_m(list(starts), list(sets), d, g, G, mk):
                    best = mk
                    break
        _, mk_opt = its.optimal_schedule(d, g, G)
        assert mk_opt == best, (d, g, G)


def _canonical_by_brute_force(d, g, G, release, now):
    """The canonical optimal schedule (reading 2) stated on schedules and found by brute force over integer start vectors:
    among the start vectors that (a) respect the capacity at every instant (GPUs count from their release time on),
    (b) reach the minimum makespan and (c) are tight -- going through the tasks in order of (start, candidate position),
    every task starts at the earliest instant, not before the task before it, at which enough GPUs are idle -- the one
    whose order (by start, then candidate position) comes first when orders are compared position by position in the
    candidate order (more GPUs first, then longer, then lower index)."""
    n = len(d)
    cand = sorted(range(n), key=lambda i: (-g[i], -d[i], i))
    cpos = {i: p for p, i in enumerate(cand)}
    horizon = int(max([now] + list(release))) + sum(d) + 1
    avail = lambda t: sum(1 for r in release if max(r, now) <= t)
    best_mk, best = None, None
    for starts in itertools.product(range(int(now), horizon), repeat=n):
        mk = max([now] + [s + di for s, di in zip(starts, d)])
        if best_mk is not None and mk > best_mk:
            continue
        if any(sum(g[i] for i in range(n) if starts[i] <= t < starts[i] + d[i]) > avail(t) for t in range(int(now), mk)):
            continue
        order = sorted(range(n), key=lambda i: (starts[i], cpos[i]))
        tight, prev = True, int(now)
        for p, i in enumerate(order):
            t = prev
            while avail(t) - sum(g[j] for j in order[:p] if starts[j] <= t < starts[j] + d[j]) < g[i]:
                t += 1
            if t != starts[i]:
                tight = False
                break
            prev = starts[i]
        if not tight:
            continue
        key = [cpos[i] for i in order]
        if best_mk is None or mk < best_mk or key < best[0]:
            best_mk, best = mk, (key, list(starts))
    return best[1], best_mk


def test_canonical_choice_equals_the_rule_stated_on_schedules():
    rng = np.random.default_rng(10)
    ties = 0
    for trial in range(60):
        n, G = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        d = [int(x) for x in rng.integers(1, 5, size=n)]
        g = [int(x) for x in rng.integers(1, G + 1, size=n)]
        release = [0] * G if trial % 3 else [int(x) for x in rng.integers(0, 4, size=G)]
        now = 0 if trial % 4 else 1
        want, mk_want = _canonical_by_brute_force(d, g, G, release, now)
        got, mk = its.optimal_schedule(d, g, G, release, now)
        assert mk == mk_want and [float(x) for x in want] == [float(x) for x in got], (d, g, G, release, now)
        ties += len(set(zip(d, g))) < n
    assert ties > 5         # instances with twin tasks, where only the order by index separates two optimal schedules
