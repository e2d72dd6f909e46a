"""The library's intra-task scheduler (host code behind the C ABI) against the oracle: identical admissions, in the same
order, on random streams of submissions and exits; the memory-model fit bit for bit."""
import numpy as np
import pytest

from oracle import admission_oracle as ad
from paper_2604_05426_amd import binding as ml


def test_memory_model_fit_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(0)
    for n in (1, 2, 5, 40):
        x = rng.choice([1, 2, 4, 8, 16, 32], size=n) * rng.integers(1, 9, size=n) * 1024.0
        y = 4.0e9 + 2.2e5 * x + rng.normal(0, 5e7, size=n)
        assert ml.memory_model_fit(x, y) == ad.fit_memory_model(x, y)
    with pytest.raises(ml.MultiLoraError):
        ml.memory_model_fit([], [])


@pytest.mark.parametrize("seed", range(10))
def test_scheduler_matches_oracle_on_random_streams(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.choice([256, 1024, 2048]))
    k0, k1 = 6.0e9, float(rng.uniform(1e5, 4e5))
    cap, margin = 288.0e9 * float(rng.uniform(0.05, 0.3)), float(rng.uniform(0.8, 1.0))
    orc = ad.Scheduler(ad.Params(k0, k1, cap, margin, L))
    lib = ml.Admission(k0, k1, cap, margin, L)
    nxt = 0
    for step in range(300):
        u = rng.random()
        if u < 0.45:
            b = int(rng.choice([1, 2, 4, 8, 16, 32]))
            orc.submit(nxt, b); lib.submit(nxt, b); nxt += 1
        elif u < 0.7:
            assert lib.fill() == orc.fill()
        elif orc.running:
            job = orc.running[int(rng.integers(len(orc.running)))][0]
            assert lib.exit(job) == orc.exit(job)
        assert lib.running() == orc.running
    assert orc.total_batch() > 0
    lib.destroy()


def test_scheduler_rejects_bad_arguments():
    with pytest.raises(ml.MultiLoraError):
        ml.Admission(0.0, 1.0, 100.0, 1.5, 8)
    s = ml.Admission(0.0, 1.0, 100.0, 1.0, 1)
    s.submit(7, 4)
    with pytest.raises(ml.MultiLoraError):
        s.submit(7, 2)                     # duplicate id
    with pytest.raises(ml.MultiLoraError):
        s.submit(8, 0)                     # batch size
    with pytest.raises(ml.MultiLoraError):
        s.exit(7)                          # pending, not running
    assert s.fill() == [7] and s.running() == [(7, 4)]
    s.destroy()
