"""Pins of the multi-step scheduling oracle (Algorithm 1 with the replay
buffer, the maximum delay d and eviction; Section 3.4, 4.2, 5.4)."""
import os

import numpy as np
import pytest

from oracle import allocation, scheduler

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LO, HI, SOLVE = 0.125, 0.75, 1.0


def test_second_round_accounting_matches_the_printed_means():
    # Section 5.4: 35.8 % / 4.5 % of the steps need a second sampling round -> 33 379 / 25 676 rollouts per step
    cost = allocation.sampling_cost("pc", 128, s=3, n_pilot=32, n_commit=96)
    assert cost == 24576
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eviction_rollouts_per_step.txt")) if l[0] != "#"]
    assert len(rows) == 2
    for _, pct, printed in rows:
        f = float(pct) / 100.0
        got = scheduler.mean_rollouts_per_step(cost, f)
        # the percentage is printed to one decimal: +-0.05 % of a round, plus the rounding of the mean itself
        assert abs(got - float(printed)) <= cost * 0.0005 + 0.5, (pct, got, printed)
        # a second round that repeated only the pilot pass would not give the printed means
        assert abs(cost + f * 3 * 128 * 32 - float(printed)) > 500


def _mk(b_t=2, d=1):
    return scheduler.Scheduler(LO, HI, SOLVE, b_t, d)


def test_hand_worked_trace():
    # worked by hand from Algorithm 1: b_t = 2, d = 1, n_pilot = 4 (p_hat in quarters)
    s = _mk()
    # step 0: keep 10, 12, 14; 11 is solved (evicted, too easy), 13 too hard
    cls, ev, cnt = s.pilot([10, 11, 12, 13, 14], [0, 1, 2, 3, 4], [0.25, 1.0, 0.5, 0.0, 0.75])
    assert cls.tolist() == [1, 2, 1, 0, 1] and ev.tolist() == [0, 1, 0, 0, 0] and cnt.tolist() == [3, 1, 1, 1]
    (u, tg, age), (au, _) = s.commit()
    assert u.tolist() == [10, 12] and tg.tolist() == [0, 2] and age.tolist() == [0, 0] and len(au) == 0
    assert s.available() == 1 and s.t == 1
    # step 1: the current survivor (22) goes first, the buffered one (14, one step old) fills the batch
    cls, ev, cnt = s.pilot([20, 21, 22], [5, 6, 7], [0.0, 1.0, 0.25])
    assert cls.tolist() == [0, 2, 1] and ev.tolist() == [0, 1, 0]
    (u, tg, age), (au, _) = s.commit()
    assert u.tolist() == [22, 14] and age.tolist() == [0, 1] and len(au) == 0 and s.available() == 0
    # step 2: four survivors, two wait
    s.pilot([30, 31, 32, 33], [0] * 4, [0.5] * 4)
    (u, _, age), (au, _) = s.commit()
    assert u.tolist() == [30, 31] and age.tolist() == [0, 0] and len(au) == 0 and s.available() == 2
    # step 3: nothing survives the pilot; the two waiting prompts are committed with delay 1
    s.pilot([40], [0], [0.0])
    (u, _, age), (au, _) = s.commit()
    assert u.tolist() == [32, 33] and age.tolist() == [1, 1] and s.available() == 0
    # steps 4, 5: 52 waits through step 5 (current survivors go first) and is then too old for d = 1
    s.pilot([50, 51, 52], [0] * 3, [0.5] * 3)
    (u, _, _), (au, _) = s.commit()
    assert u.tolist() == [50, 51] and len(au) == 0
    s.pilot([60, 61, 62], [0] * 3, [0.5] * 3)
    (u, _, age), (au, atg) = s.commit()
    assert u.tolist() == [60, 61] and age.tolist() == [0, 0] and au.tolist() == [52] and s.available() == 1
    # step 6: an empty sampling batch; the batch stays short
    s.pilot([], [], [])
    (u, _, age), (au, _) = s.commit()
    assert u.tolist() == [62] and age.tolist() == [1] and s.available() == 0
    st = s.stats
    assert st["short_steps"] == 1 and st["committed"] == 13 and st["aged_out"] == 1 and st["buffered"] == 14
    assert st["evictions"] == 2 and s.is_evicted([11, 21, 10, 99]).tolist() == [1, 1, 0, 0] and s.t == 7


def test_zero_delay_is_the_single_step_rule():
    # d = 0: nothing can wait, so every step is the one-step filter + cap of Section 3.3
    rng = np.random.default_rng(5)
    s = scheduler.Scheduler(LO, HI, SOLVE, 7, 0)
    for step in range(40):
        n = int(rng.integers(0, 30))
        ph = (rng.integers(0, 9, n) / 8.0).astype(np.float32)
        uids = np.arange(n) + 1000 * step
        cls, ev, cnt = s.pilot(uids, uids * 2, ph)
        wcls, wev, wcommit, wsurplus, wcnt = allocation.select_commit(ph, LO, HI, SOLVE, 7)
        assert np.array_equal(cls, wcls) and np.array_equal(ev, wev)
        (u, tg, age), (au, atg) = s.commit()
        assert np.array_equal(u, uids[wcommit]) and np.array_equal(tg, 2 * uids[wcommit]) and not age.any()
        assert np.array_equal(au, uids[wsurplus]) and s.available() == 0


@pytest.mark.parametrize("b_t,d", [(4, 4), (16, 2), (3, 7), (1, 1)])
def test_invariants_on_random_traces(b_t, d):
    rng = np.random.default_rng(b_t * 100 + d)
    s = scheduler.Scheduler(LO, HI, SOLVE, b_t, d)
    stamp, left = {}, {}
    uid = 0
    for step in range(200):
        for _ in range(int(rng.integers(1, 3))):
            n = int(rng.integers(0, 3 * b_t + 1))
            ph = (rng.integers(0, 9, n) / 8.0).astype(np.float32)
            uids = np.arange(uid, uid + n)
            uid += n
            cls, ev, cnt = s.pilot(uids, uids, ph)
            for q in range(n):
                if cls[q] == scheduler.KEEP:
                    stamp[int(uids[q])] = step
                assert ev[q] == (ph[q] >= 1.0)
            cur = [int(x) for x in uids[cls == scheduler.KEEP]]
        before = s.available()
        (u, tg, age), (au, atg) = s.commit()
        assert len(u) == min(b_t, before)
        assert (age >= 0).all() and (age <= d).all()
        for x, a in zip(u.tolist(), age.tolist()):
            assert stamp[x] == step - a and x not in left
            left[x] = "committed"
        for x in au.tolist():
            assert step + 1 - stamp[x] > d and x not in left
            left[x] = "aged"
        # survivors of this step come before older ones; older ones oldest first
        ages = age.tolist()
        zeros = [a == 0 for a in ages]
        assert zeros == sorted(zeros, reverse=True)
        tail = [a for a in ages if a > 0]
        assert tail == sorted(tail, reverse=True)
        st = s.stats
        assert st["buffered"] == st["committed"] + st["aged_out"] + s.available()
    assert s.stats["aged_out"] + s.stats["short_steps"] > 0 and s.stats["multi_round_steps"] > 0
