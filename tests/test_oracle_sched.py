"""Pins for the oracle's VLT and LVF (paper Sections 4.2.1 and 4.2.2): a
hand-worked run of Algorithm 1, the shape of the VLT curves the paper describes,
and properties every LVF decision must have."""
import numpy as np
import pytest

from oracle import kv_oracle as O
from tests import schedfixture

PAPER = (3.0, 0.0, 0.5, 0.1, 5.0)     # alpha, beta_B, beta_F, S_B (between tokens), S_F (first token)


def test_hand_worked_example():
    params, reqs, t_now, vlt, cases = schedfixture.load()
    for r, want in zip(reqs, vlt):
        assert O.sched_vlt(params, r, t_now) == pytest.approx(want, abs=1e-12)
    for c in cases:
        rc, pre, pri, fcfs = O.sched_lvf(params, reqs, t_now, c["b_xfer"], c["b_hbm"])
        assert rc == O.OK
        assert (pre, pri, fcfs) == (c["preempt"], c["prioritize"], c["fcfs"])


def test_vlt_curves():
    """Section 4.2.1: running requests are negative and fall as they run; waiting
    and rotary ones stay at zero within tolerance, then rise linearly, rotary ones
    alpha times as fast."""
    a, bb, bf, sb, sf = 2.5, 1.5, 0.25, 0.2, 4.0
    p = (a, bb, bf, sb, sf)
    for dt in [0.0, 0.1, 0.29, 0.3, 0.31, 1.0, 7.5]:
        assert O.sched_vlt(p, (0, O.RUNNING, 1, 10.0), 10.0 + dt) == pytest.approx(-dt)
        assert O.sched_vlt(p, (0, O.ROTARY, 1, 10.0), 10.0 + dt) == pytest.approx(a * max(0.0, dt - bb * sb))
        assert O.sched_vlt(p, (0, O.WAITING, 1, 10.0), 10.0 + dt) == pytest.approx(max(0.0, dt - bf * sf))
    # negative tolerance coefficients are allowed (beta in R): lag starts before time zero
    assert O.sched_vlt((1.0, -1.0, -1.0, 0.5, 2.0), (0, O.ROTARY, 1, 5.0), 5.0) == pytest.approx(0.5)
    assert O.sched_vlt((1.0, -1.0, -1.0, 0.5, 2.0), (0, O.WAITING, 1, 5.0), 5.0) == pytest.approx(2.0)
    # alpha = 0 silences rotary requests entirely
    assert O.sched_vlt((0.0, 0.0, 0.0, 0.1, 1.0), (0, O.ROTARY, 1, 0.0), 99.0) == 0.0


def random_case(rng, n):
    reqs = []
    for i in range(n):
        st = int(rng.integers(0, 3))
        reqs.append((i, st, int(rng.integers(0, 12)), float(np.round(rng.uniform(80, 100), 1))))
    return reqs


def test_lvf_properties_on_random_queues():
    rng = np.random.default_rng(3)
    seen_fcfs = seen_lvf = 0
    for _ in range(3000):
        reqs = random_case(rng, int(rng.integers(0, 12)))
        b_xfer, b_hbm = int(rng.integers(0, 30)), int(rng.integers(0, 30))
        t_now = 100.0
        rc, pre, pri, fcfs = O.sched_lvf(PAPER, reqs, t_now, b_xfer, b_hbm)
        assert rc == O.OK
        by_id = {r[0]: r for r in reqs}
        vlt = {r[0]: O.sched_vlt(PAPER, r, t_now) for r in reqs}
        inactive = [r for r in reqs if r[1] != O.RUNNING]
        need = sum(r[2] for r in inactive)
        assert len(set(pre)) == len(pre) and len(set(pri)) == len(pri)
        assert all(by_id[i][1] == O.RUNNING for i in pre)          # only running requests are preempted
        assert all(by_id[i][1] != O.RUNNING for i in pri)          # only waiting / rotary are prioritised
        if b_hbm >= need:                                          # step 1: fallback
            assert fcfs and pre == []
            assert sorted(pri) == sorted(r[0] for r in inactive)
            keys = [(by_id[i][3], i) for i in pri]
            assert keys == sorted(keys)
            seen_fcfs += 1
            continue
        seen_lvf += 1
        assert not fcfs
        used = sum(by_id[i][2] for i in pri)
        assert used <= b_hbm + b_xfer                              # step 3 never overdraws the budget
        # chosen in descending VLT order, and nobody with VLT >= 0 that still fitted was skipped
        v = [vlt[i] for i in pri]
        assert v == sorted(v, reverse=True)
        left = b_hbm + b_xfer
        order = sorted(reqs, key=lambda r: (-vlt[r[0]], r[0]))
        for r in order:
            if r[1] != O.RUNNING and vlt[r[0]] >= 0 and r[2] <= left:
                assert r[0] in pri
                left -= r[2]
            else:
                assert r[0] not in pri
        # step 4: preempted requests are the most advanced running ones, and just enough of them
        swap = b_xfer - left
        freed = 0
        lagging = sorted([r for r in reqs if r[1] == O.RUNNING and vlt[r[0]] < 0], key=lambda r: (vlt[r[0]], -r[0]))
        assert pre == [r[0] for r in lagging[:len(pre)]]           # from the tail of the sorted list
        for k, i in enumerate(pre):
            assert swap - freed > 0                                # each one was still needed
            freed += by_id[i][2]
        assert freed >= swap or len(pre) == len(lagging)           # enough, or nobody left to preempt
    assert seen_fcfs > 100 and seen_lvf > 100


def test_lvf_bad_arguments():
    assert O.sched_lvf(PAPER, [(0, 3, 1, 0.0)], 1.0, 1, 1)[0] == O.EINVAL       # unknown state
    assert O.sched_lvf(PAPER, [(0, 0, -1, 0.0)], 1.0, 1, 1)[0] == O.EINVAL      # negative block count
    assert O.sched_lvf(PAPER, [(0, 0, 1, 0.0)], 1.0, -1, 1)[0] == O.EINVAL
    rc, pre, pri, fcfs = O.sched_lvf(PAPER, [], 1.0, 5, 5)
    assert (rc, pre, pri, fcfs) == (O.OK, [], [], True)
