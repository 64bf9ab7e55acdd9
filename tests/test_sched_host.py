"""The library's VLT / LVF (host code, no GPU) against the paper-derived worked
example and against the oracle on random queues."""
import numpy as np
import pytest

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from tests import schedfixture


def test_worked_example():
    params, reqs, t_now, vlt, cases = schedfixture.load()
    for r, want in zip(reqs, vlt):
        assert B.kv_sched_vlt(params, r, t_now) == pytest.approx(want, abs=1e-12)
    for c in cases:
        rc, pre, pri, fcfs = B.kv_sched_lvf(params, reqs, t_now, c["b_xfer"], c["b_hbm"])
        assert (rc, pre, pri, fcfs) == (0, c["preempt"], c["prioritize"], c["fcfs"])


def test_same_decisions_as_the_oracle():
    rng = np.random.default_rng(11)
    kinds = set()
    for _ in range(4000):
        params = (float(rng.choice([0, 1, 3, 4.5])), float(rng.uniform(-1, 2)), float(rng.uniform(-1, 2)),
                  float(rng.choice([0.05, 0.1, 0.5])), float(rng.choice([1.0, 5.0])))
        n = int(rng.integers(0, 14))
        # coarse times and VLT ties on purpose
        reqs = [(i, int(rng.integers(0, 3)), int(rng.integers(0, 10)), float(rng.integers(90, 101)))
                for i in rng.permutation(n)]
        b_xfer, b_hbm = int(rng.integers(0, 25)), int(rng.integers(0, 25))
        want = O.sched_lvf(params, reqs, 100.0, b_xfer, b_hbm)
        got = B.kv_sched_lvf(params, reqs, 100.0, b_xfer, b_hbm)
        assert got == want
        for r in reqs:
            assert B.kv_sched_vlt(params, r, 100.0) == O.sched_vlt(params, r, 100.0)
        kinds.add((want[3], bool(want[1]), bool(want[2])))
    assert len(kinds) >= 5
    assert B.kv_sched_lvf((1, 0, 0, 1, 1), [(0, 5, 1, 0.0)], 1.0, 1, 1)[0] == B.KV_EINVAL
    assert B.kv_sched_lvf((1, 0, 0, 1, 1), [(0, 0, 1, 0.0)], 1.0, 1, -2)[0] == B.KV_EINVAL
