"""CPU oracle for the dynamic inter-task scheduler -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Sec. 6.2 ("Dynamic Inter-Task Scheduling"): n tasks with profiled durations d_i and GPU requirements
g_i on G GPUs, every task holds its g_i GPUs for its whole duration, minimise the makespan C_max (the problem
P | size_j | C_max); the paper states it as a constraint program over start times s_i, GPU assignments x_ig, pair orders
y_ij and C_max with disjunctive no-overlap constraints per shared GPU, and re-plans on every task arrival and completion.

What this file holds, slow and plain:

* ``check_schedule``   the paper's constraints written out: sum_g x_ig = g_i; two tasks that share a GPU do not overlap
                       in time; nobody starts before `now` or before an assigned GPU is released.
* ``time_indexed_optimum``  brute force straight on that definition for small integer data: every combination of
                       integer start times up to a horizon, capacity checked instant by instant.
* ``optimal_schedule`` the exact optimum by enumeration of task lists, each list turned into a schedule by starting
                       its tasks in list order, each as early as possible but not before the one before it (every
                       schedule in which no task can start earlier with the others left alone is the schedule of
                       its own tasks listed by start time, and some such schedule is optimal).
* ``Cluster``          the event loop: arrival and completion re-plan; ``poll`` starts what the plan says is due.

Readings where the paper is silent:
  1. GPUs are interchangeable, so a set of start times is feasible iff at every instant the tasks running need at most
     the GPUs then available (GPUs still held by earlier work count as unavailable until their release time); concrete
     GPUs are then handed out in order of start time, lowest free index first.  (Intervals: a demand-feasible set of
     intervals can always be coloured this way.)
  2. Several schedules reach the optimum.  The canonical one: candidate order = tasks sorted by (g descending,
     d descending, index ascending); lists are enumerated depth first in that candidate order, tasks with equal (d, g)
     only in index order, tasks that come out with equal start times only in candidate order (other lists repeat a
     schedule); the first list whose schedule attains the minimum (strict improvement replaces the incumbent) is the
     answer.  The library must return exactly this schedule.
  3. Re-planning keeps running tasks where they are: a GPU held by a running task is released at that task's estimated
     end (start + d), or `now` if that estimate has already passed.
  4. ``poll(now)`` starts, in order of planned start (ties in candidate order), every pending task whose planned start
     is <= now and for which g_i GPUs are actually idle; a task started late, or one that cannot start because a
     running task has overrun its estimate, makes the remaining plan stale, so poll re-plans after it has started
     what it could whenever that happened.
  5. Times are fp64; two times closer than 1e-9 count as equal.
"""
from __future__ import annotations

import itertools
from typing import Dict, List, Optional, Sequence, Tuple

EPS = 1e-9


def list_schedule(order: Sequence[int], d, g, G: int, release: Optional[Sequence[float]] = None, now: float = 0.0):
    """Tasks are started in the order of the list, none before the one listed before it: each at the earliest time, not
    before the previous start, at which g_i GPUs are idle (GPUs are only ever taken from a start time on, so "idle at s"
    means idle for good).  Returns ({task: start}, makespan of the listed tasks)."""
    free = [max(float(r), now) for r in release] if release is not None else [now] * G
    front = now
    starts: Dict[int, float] = {}
    for i in order:
        need = int(g[i])
        by_time = sorted(range(G), key=lambda q: (free[q], q))
        s = max(front, free[by_time[need - 1]])
        for q in by_time[:need]:
            free[q] = s + float(d[i])
        front = s
        starts[i] = s
    makespan = max([now] + [starts[i] + float(d[i]) for i in order])
    return starts, makespan


def candidate_order(d, g) -> List[int]:
    return sorted(range(len(d)), key=lambda i: (-int(g[i]), -float(d[i]), i))


def optimal_schedule(d, g, G: int, release: Optional[Sequence[float]] = None, now: float = 0.0):
    """(starts list, makespan) of the canonical optimal schedule (reading 2).  Plain enumeration: fine up to ~8 tasks."""
    n = len(d)
    for i in range(n):
        if not (1 <= int(g[i]) <= G) or not float(d[i]) > 0.0:
            raise ValueError("bad task")
    cand = candidate_order(d, g)
    pos_of = {i: p for p, i in enumerate(cand)}
    best = (None, float("inf"))

    def rec(prefix: List[int], left: List[int]):
        nonlocal best
        if not left:
            starts, mk = list_schedule(prefix, d, g, G, release, now)
            for p in range(n - 1):
                a, b = prefix[p], prefix[p + 1]
                if abs(starts[b] - starts[a]) <= EPS and pos_of[b] < pos_of[a]:
                    return    # equal starts out of candidate order: the same schedule comes up under another list
            if mk < best[1] - EPS:
                best = ([starts[i] for i in range(n)], mk)
            return
        for pos, i in enumerate(left):
            # equal tasks only in index order: an earlier-listed twin still waiting forbids this one
            if any(float(d[j]) == float(d[i]) and int(g[j]) == int(g[i]) for j in left[:pos]):
                continue
            rec(prefix + [i], left[:pos] + left[pos + 1:])

    rec([], cand)
    if n == 0:
        return [], now
    return best


def assign_gpus(starts, d, g, G: int, release: Optional[Sequence[float]] = None, now: float = 0.0) -> List[List[int]]:
    """Concrete GPUs, handed out in order of start time (ties: candidate order), lowest free index first (reading 1)."""
    release = list(release) if release is not None else [now] * G
    free_at = list(release)
    cand_pos = {i: p for p, i in enumerate(candidate_order(d, g))}
    out: List[List[int]] = [[] for _ in starts]
    for i in sorted(range(len(starts)), key=lambda i: (starts[i], cand_pos[i])):
        mine = [q for q in range(G) if free_at[q] <= starts[i] + EPS][: int(g[i])]
        if len(mine) < int(g[i]):
            raise ValueError("start times are not demand-feasible")
        for q in mine:
            free_at[q] = starts[i] + float(d[i])
        out[i] = mine
    return out


def check_schedule(starts, gpus, d, g, G: int, release: Optional[Sequence[float]] = None, now: float = 0.0) -> float:
    """The constraints of the paper's program; returns the makespan, raises AssertionError on a violation."""
    release = list(release) if release is not None else [now] * G
    n = len(starts)
    for i in range(n):
        assert len(set(gpus[i])) == len(gpus[i]) == int(g[i]), f"task {i}: sum_g x_ig != g_i"
        assert all(0 <= q < G for q in gpus[i])
        assert starts[i] >= now - EPS
        for q in gpus[i]:
            assert starts[i] >= release[q] - EPS, f"task {i} starts before GPU {q} is released"
    for i in range(n):
        for j in range(i + 1, n):
            if set(gpus[i]) & set(gpus[j]):
                assert starts[i] + float(d[i]) <= starts[j] + EPS or starts[j] + float(d[j]) <= starts[i] + EPS, \
                    f"tasks {i} and {j} share a GPU and overlap"
    return max([now] + [starts[i] + float(d[i]) for i in range(n)])


def check_big_m(starts, gpus, d, g, G: int, c_max: float) -> bool:
    """The paper's program (Sec. 6.2) evaluated as printed, for given start times s_i and GPU sets (x_ig = 1 iff q in
    gpus[i]):  sum_g x_ig = g_i and s_i + d_i <= C_max for every task, and for every pair i < j some y_ij in {0, 1} with,
    for EVERY GPU q,
        s_i + d_i <= s_j + M (3 - x_iq - x_jq - y_ij)       and       s_j + d_j <= s_i + M (2 - x_iq - x_jq + y_ij),
    M = sum_i d_i.  (One y_ij per pair serves all GPUs, as the paper notes.)  M = sum d is large enough to switch a
    constraint off only for schedules whose tasks all end by M -- which every schedule worth considering does, since
    running the tasks one after another already ends at M; a schedule that ends later is rejected here although it may
    satisfy the plain no-overlap statement.  True iff all constraints hold."""
    n = len(starts)
    M = float(sum(float(x) for x in d))
    x = [[1 if q in gpus[i] else 0 for q in range(G)] for i in range(n)]
    for i in range(n):
        if sum(x[i]) != int(g[i]) or len(set(gpus[i])) != len(gpus[i]):
            return False
        if starts[i] < 0.0 or starts[i] + float(d[i]) > c_max + EPS:
            return False
    for i in range(n):
        for j in range(i + 1, n):
            ok_pair = False
            for y in (0, 1):
                if all(starts[i] + float(d[i]) <= starts[j] + M * (3 - x[i][q] - x[j][q] - y) + EPS and
                       starts[j] + float(d[j]) <= starts[i] + M * (2 - x[i][q] - x[j][q] + y) + EPS for q in range(G)):
                    ok_pair = True
            if not ok_pair:
                return False
    return True


def time_indexed_optimum(d: Sequence[int], g: Sequence[int], G: int, horizon: int) -> int:
    """Minimum makespan over all integer start vectors in [0, horizon), demand checked at every integer instant."""
    n = len(d)
    best = None
    for starts in itertools.product(range(horizon), repeat=n):
        mk = max(s + di for s, di in zip(starts, d))
        if best is not None and mk >= best:
            continue
        ok = True
        for t in range(mk):
            if sum(gi for s, di, gi in zip(starts, d, g) if s <= t < s + di) > G:
                ok = False
                break
        if ok:
            best = mk
    return best


class Cluster:
    """Event-driven re-planning (readings 3, 4)."""

    def __init__(self, G: int):
        self.G = G
        self.pending: Dict[int, Tuple[float, int]] = {}          # id -> (d, g), insertion order = submission order
        self.running: Dict[int, Tuple[float, float, List[int]]] = {}   # id -> (start, estimated end, gpus)
        self.plan: Dict[int, float] = {}                         # pending id -> planned start
        self.planned_makespan = 0.0
        self.next_id = 0

    def _release(self, now: float) -> List[float]:
        rel = [now] * self.G
        for s, e, gpus in self.running.values():
            for q in gpus:
                rel[q] = max(e, now)
        return rel

    def _replan(self, now: float) -> None:
        ids = list(self.pending)
        d = [self.pending[i][0] for i in ids]
        g = [self.pending[i][1] for i in ids]
        rel = self._release(now)
        starts, mk = optimal_schedule(d, g, self.G, rel, now)
        self.plan = {ids[p]: starts[p] for p in range(len(ids))}
        self.planned_makespan = max([mk] + [r for r in rel])

    def submit(self, now: float, duration: float, gpus: int) -> int:
        if not (1 <= gpus <= self.G) or not duration > 0.0:
            raise ValueError("bad task")
        tid = self.next_id
        self.next_id += 1
        self.pending[tid] = (float(duration), int(gpus))
        self._replan(now)
        return tid

    def complete(self, now: float, tid: int) -> None:
        if tid not in self.running:
            raise KeyError(tid)
        del self.running[tid]
        self._replan(now)

    def poll(self, now: float) -> List[Tuple[int, List[int]]]:
        ids = list(self.pending)
        d = [self.pending[i][0] for i in ids]
        g = [self.pending[i][1] for i in ids]
        cand_pos = {ids[i]: p for p, i in enumerate(candidate_order(d, g))}
        due = sorted((t for t in ids if self.plan[t] <= now + EPS), key=lambda t: (self.plan[t], cand_pos[t]))
        busy = set(q for s, e, gpus in self.running.values() for q in gpus)
        started: List[Tuple[int, List[int]]] = []
        stale = False
        for t in due:
            dur, need = self.pending[t]
            idle = [q for q in range(self.G) if q not in busy][:need]
            if len(idle) < need:
                stale = True          # somebody has overrun the estimate
                continue
            if self.plan[t] < now - EPS:
                stale = True          # started late: everything planned behind it moves
            busy.update(idle)
            self.running[t] = (now, now + dur, idle)
            del self.pending[t]
            started.append((t, idle))
        if stale:
            self._replan(now)
        else:
            for t, _ in started:
                del self.plan[t]
        return started
