"""Pins for the intra-task scheduler oracle (paper Sec. 6.1, App. "Intra-Task Scheduling Details"): the fitted memory
model against closed forms and the library least-squares fit, hand-worked admission / backfill sequences, and the
invariants of the greedy policy on random job streams."""
import numpy as np
import pytest

from oracle import admission_oracle as ad


def test_memory_model_fit():
    BL = np.array([256., 512., 1024., 2048., 4096.])
    k0, k1 = ad.fit_memory_model(BL, 3.0e9 + 1.5e6 * BL)              # points on an exact line
    assert k0 == pytest.approx(3.0e9, rel=1e-12) and k1 == pytest.approx(1.5e6, rel=1e-12)
    rng = np.random.default_rng(0)
    y = 2.0e9 + 9.0e5 * BL + rng.normal(0, 1e7, size=5)
    k0, k1 = ad.fit_memory_model(BL, y)
    p1, p0 = np.polyfit(BL, y, 1)
    assert k0 == pytest.approx(p0, rel=1e-9) and k1 == pytest.approx(p1, rel=1e-9)
    # residuals of a least-squares line sum to zero and are orthogonal to x
    res = y - (k0 + k1 * BL)
    assert abs(res.sum()) < 1e-3 and abs((res * BL).sum()) < 10.0
    assert ad.fit_memory_model([512., 512.], [1.0e9, 3.0e9]) == (2.0e9, 0.0)     # no spread in x: a constant


def _sched(capacity_batches, L=256):
    # k0 = 0, k1 = 1 / L: Mhat(B) = B, so "capacity" is simply a total batch size
    return ad.Scheduler(ad.Params(k0=0.0, k1=1.0 / L, capacity=float(capacity_batches), margin=1.0, seq_len=L))


def test_greedy_admission_in_decreasing_batch_size():
    s = _sched(10)
    for job, b in enumerate([1, 4, 2, 4, 8, 1]):
        s.submit(job, b)
    # order tried: 8 (job 4) fits -> B = 8; 4 (job 1), 4 (job 3) do not fit; 2 (job 2) fits -> 10; 1s do not fit
    assert s.fill() == [4, 2] and s.total_batch() == 10
    assert [j for j, _ in s.pending] == [0, 1, 3, 5]


def test_backfill_prefers_the_same_batch_size_then_anything_that_fits():
    s = _sched(8)
    for job, b in enumerate([4, 4, 4, 2, 1, 1]):
        s.submit(job, b)
    assert s.fill() == [0, 1]                                 # 4 + 4 = 8
    assert s.exit(0) == [2]                                   # the pending 4 takes the slot although 2 and 1 are older ... smaller
    assert s.exit(1) == [3, 4, 5]                             # no 4 left: 2, then 1, 1 (decreasing size), B = 4 + 2 + 1 + 1
    assert s.total_batch() == 8 and [j for j, _ in s.running] == [2, 3, 4, 5]
    assert s.exit(3) == []                                    # nothing pending
    with pytest.raises(ValueError):
        s.exit(3)


def test_margin_and_offset_enter_the_fit_test():
    # Mhat(B) = 1000 + 10 B L with L = 2, capacity 2000, margin 0.9: B <= 40
    s = ad.Scheduler(ad.Params(k0=1000.0, k1=10.0, capacity=2000.0, margin=0.9, seq_len=2))
    s.submit(0, 32); s.submit(1, 8); s.submit(2, 1)
    assert s.fill() == [0, 1] and s.total_batch() == 40       # exactly at the margin counts as fitting (<=)
    assert not s.fits(1)


@pytest.mark.parametrize("seed", range(8))
def test_invariants_on_random_streams(seed):
    rng = np.random.default_rng(seed)
    cap = int(rng.integers(8, 64))
    s = _sched(cap)
    nxt = 0
    for step in range(200):
        if rng.random() < 0.5:
            s.submit(nxt, int(rng.choice([1, 2, 4, 8, 16, 32]))); nxt += 1
            before = list(s.running)
            adm = s.fill()
        elif s.running:
            victim = s.running[int(rng.integers(len(s.running)))]
            same_waiting = [j for j, b in s.pending if b == victim[1]]
            before = [e for e in s.running if e != victim]
            adm = s.exit(victim[0])
            if same_waiting:                                   # a same-size job always fits the slot it replaces
                assert adm[0] == same_waiting[0]
        else:
            continue
        assert s.total_batch() <= cap                                         # never over capacity
        assert all(not s.fits(b) for _, b in s.pending)                       # saturated: nothing pending fits
        assert s.running[:len(before)] == before                              # admission order is kept
        assert [j for j, _ in s.running[len(before):]] == adm
