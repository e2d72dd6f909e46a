"""CPU oracle for the online greedy intra-task scheduler -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Sec. 6.1 and App. "Intra-Task Scheduling Details":

* memory model: the profiled points (B L, peak bytes) are fitted by least squares to  Mhat(B) = k0 + k1 B L
  (B = total batch size of the co-located adapters, L = sequence length);
* admission: pending jobs are taken in decreasing per-adapter batch size; a job is admitted only if
  Mhat(B_current + b_new) stays within the safety margin of the capacity; this goes on until no pending job fits;
* backfill: when a job exits, a pending job of the same batch size is preferred for the vacated slot; when there is none
  (or it does not fit) jobs of other batch sizes are admitted if the model says the mixed configuration fits.

Readings where the paper is silent:
  1. Jobs of equal batch size are taken in submission order.
  2. A job that does not fit is skipped, not waited for: smaller jobs behind it may still be admitted ("until no further
     admission is feasible").
  3. "Fits" means  k0 + k1 (B_current + b) L <= margin x capacity  (margin in (0, 1]).
  4. After an exit: first one pending job of the same batch size (the oldest) if it fits, then the ordinary greedy pass
     over everything still pending - freed memory is never left idle while some pending job fits.
  5. The running set is reported in admission order; that order is the segment order of the next step's batch.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple


def fit_memory_model(BL: Sequence[float], peak: Sequence[float]) -> Tuple[float, float]:
    """Least-squares line peak = k0 + k1 * BL:  k1 = sum (x - xbar)(y - ybar) / sum (x - xbar)^2,  k0 = ybar - k1 xbar,
    sums left to right in fp64 (the scheduler compares the model with a capacity, so the formula is part of the
    definition).  All x equal: k1 = 0, k0 = ybar."""
    n = len(BL)
    if n == 0:
        raise ValueError("no profiling points")
    xbar = ybar = 0.0
    for x, y in zip(BL, peak):
        xbar += float(x); ybar += float(y)
    xbar /= n; ybar /= n
    num = den = 0.0
    for x, y in zip(BL, peak):
        num += (float(x) - xbar) * (float(y) - ybar)
        den += (float(x) - xbar) * (float(x) - xbar)
    k1 = num / den if den > 0.0 else 0.0
    return ybar - k1 * xbar, k1


@dataclass
class Params:
    k0: float
    k1: float
    capacity: float
    margin: float
    seq_len: int


class Scheduler:
    def __init__(self, p: Params):
        self.p = p
        self.pending: List[Tuple[int, int]] = []      # (job, batch size) in submission order
        self.running: List[Tuple[int, int]] = []      # in admission order

    def total_batch(self) -> int:
        return sum(b for _, b in self.running)

    def fits(self, b: int) -> bool:
        p = self.p
        return p.k0 + p.k1 * float(self.total_batch() + b) * float(p.seq_len) <= p.margin * p.capacity

    def submit(self, job: int, batch: int) -> None:
        if batch < 1 or any(j == job for j, _ in self.pending + self.running):
            raise ValueError("bad job")
        self.pending.append((job, batch))

    def _admit(self, entry) -> None:
        self.pending.remove(entry)
        self.running.append(entry)

    def fill(self) -> List[int]:
        """Greedy admission in decreasing batch size (submission order within a size)."""
        admitted = []
        order = sorted(range(len(self.pending)), key=lambda i: (-self.pending[i][1], i))
        for entry in [self.pending[i] for i in order]:
            if self.fits(entry[1]):
                self._admit(entry)
                admitted.append(entry[0])
        return admitted

    def exit(self, job: int) -> List[int]:
        """The job leaves (early exit or completion); returns the jobs admitted in its place."""
        hit = [e for e in self.running if e[0] == job]
        if not hit:
            raise ValueError("job is not running")
        self.running.remove(hit[0])
        b = hit[0][1]
        admitted = []
        same = [e for e in self.pending if e[1] == b]
        if same and self.fits(b):
            self._admit(same[0])
            admitted.append(same[0][0])
        return admitted + self.fill()
