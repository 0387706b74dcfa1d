"""The library's host-side scheduler (pc_sched_*) against the oracle's
Algorithm 1 loop, call by call and bit-exact, on synthetic multi-epoch runs
in which the prompts get easier as training proceeds (the paper's regime:
Section 3.3, "prompts become easier over the course of training").  Host
code only: no GPU needed."""
import numpy as np
import pytest

from oracle import allocation, scheduler as osched

LO, HI, SOLVE = 0.125, 0.75, 1.0


def _lib_sched(*a):
    from paper_2605_26606_amd import Scheduler
    return Scheduler(*a)


def _drifting_run(b_t, d, s_factor, n_pilot, n_prompts, epochs, seed, drift, second_round=True, informative=1.0):
    """Feeds both schedulers the same synthetic training run and compares every output."""
    rng = np.random.default_rng(seed)
    p_q = np.sin(0.5 * np.pi * rng.random(n_prompts)) ** 2          # Beta(1/2, 1/2) success probabilities
    # only a share of the prompts is informative at all; the rest is hopeless or trivially solved
    dull = rng.random(n_prompts) >= informative
    p_q = np.where(dull, np.where(rng.random(n_prompts) < 0.5, 0.0005, 0.9995), p_q)
    uids = np.arange(n_prompts, dtype=np.int64) * 7 + 3
    want, got = osched.Scheduler(LO, HI, SOLVE, b_t, d), _lib_sched(LO, HI, SOLVE, b_t, d)
    b_g = s_factor * b_t
    steps = 0
    for _ in range(epochs):
        ev = got.evicted(uids)
        assert np.array_equal(ev, want.is_evicted(uids))
        pool = rng.permutation(np.nonzero(ev == 0)[0])
        pos = 0
        while pos < len(pool):
            rounds = 0
            while pos < len(pool) and rounds < (2 if second_round else 1):
                batch = pool[pos:pos + b_g]
                pos += len(batch)
                p_hat = (rng.binomial(n_pilot, p_q[batch]) / np.float32(n_pilot)).astype(np.float32)
                tags = (batch.astype(np.int64) << 20) + steps
                w = want.pilot(uids[batch], tags, p_hat)
                g = got.pilot(uids[batch], tags, p_hat)
                for a, b in zip(w, g):
                    assert a.dtype == b.dtype and np.array_equal(a, b)
                rounds += 1
                if want.available() >= b_t:
                    break
            (wu, wt, wa), (wau, wat) = want.commit()
            (gu, gt, ga), (gau, gat) = got.commit()
            assert np.array_equal(wu, gu) and np.array_equal(wt, gt) and np.array_equal(wa, ga)
            assert np.array_equal(wau, gau) and np.array_equal(wat, gat)
            steps += 1
            p_q = np.minimum(1.0, p_q + drift)                      # the policy improves
            st = got.stats()
            assert st["step"] == want.t and st["buffered_now"] == want.available()
            for k, v in want.stats.items():
                assert st[k] == v, k
    return want, got, steps


@pytest.mark.parametrize("b_t,d,s,n_pilot", [(128, 4, 3, 32), (16, 4, 3, 8), (8, 0, 3, 4), (5, 2, 1, 4), (1, 1, 2, 16)])
def test_library_scheduler_follows_the_oracle(b_t, d, s, n_pilot):
    want, got, steps = _drifting_run(b_t, d, s, n_pilot, n_prompts=40 * b_t, epochs=3, seed=b_t + d, drift=0.004)
    st = got.stats()
    assert steps > 20 and st["committed"] > 0 and st["evictions"] > 0
    assert st["buffered"] == st["committed"] + st["aged_out"] + st["buffered_now"]
    got.close()


def test_eviction_shrinks_later_epochs_and_second_rounds_are_counted():
    # the paper's setting (b_t 128, s 3, n_pilot 32, d 4): solved prompts leave the pool, so later epochs are shorter
    want, got, _ = _drifting_run(128, 4, 3, 32, n_prompts=12000, epochs=3, seed=1, drift=0.002, informative=0.4)
    st = got.stats()
    assert st["evictions"] > 0 and got.evicted(np.arange(12000, dtype=np.int64) * 7 + 3).sum() > 0
    assert st["multi_round_steps"] > 0
    # cost accounting of Section 4.3 / 5.4 with the measured share of two-round steps
    cost = allocation.sampling_cost("pc", 128, s=3, n_pilot=32, n_commit=96)
    f = st["multi_round_steps"] / st["step"]
    assert cost <= osched.mean_rollouts_per_step(cost, f) <= 2 * cost
    got.close()


def test_argument_checks():
    from paper_2605_26606_amd import binding
    lib = binding.library()
    assert lib.pc_sched_create(None, None) == -1
    with pytest.raises(binding.PcError):
        _lib_sched(LO, HI, SOLVE, 0, 4)
    with pytest.raises(binding.PcError):
        _lib_sched(LO, HI, SOLVE, 4, -1)
    with pytest.raises(binding.PcError):
        _lib_sched(0.9, 0.5, SOLVE, 4, 1)
    s = _lib_sched(LO, HI, SOLVE, 2, 0)
    assert lib.pc_sched_pilot(s.handle, None, None, None, 3, None, None, None) == -1
    assert lib.pc_sched_pilot(s.handle, None, None, None, 0, None, None, None) == 0
    # an age-out buffer that is too small is refused and leaves the state as it was
    s.pilot([1, 2, 3, 4, 5], None, [0.5] * 5)
    out = np.zeros(2, np.int64)
    k = np.zeros(1, np.int32)
    assert lib.pc_sched_commit(s.handle, out.ctypes.data, None, None, k.ctypes.data, out.ctypes.data, None, 1,
                               k.ctypes.data) == -1
    assert s.stats()["buffered_now"] == 5 and s.stats()["step"] == 0
    (u, t, a), (au, at) = s.commit()
    assert u.tolist() == [1, 2] and au.tolist() == [3, 4, 5] and t.tolist() == [0, 0]
    s.close()
