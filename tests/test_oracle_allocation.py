"""Pins for oracle.allocation: Eq. 3 closed forms for binary rewards, the
filter's truth table, brute force, the advantage invariants of Section 3.2
and the per-step rollout counts the paper prints."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import allocation as al


def _binary_group(n, k):
    r = np.zeros(n, np.float32)
    r[:k] = 1.0
    return r


@pytest.mark.parametrize("n", [1, 4, 8, 16, 32])
def test_binary_stats_closed_form(n):
    # p_hat = k/n, Var = p(1-p) = k(n-k)/n^2 (Section 3.3)
    for k in range(n + 1):
        r = np.random.default_rng(k).permutation(_binary_group(n, k))
        n_pos, n_tot, mean, var = al.group_stats(r, [0, n])
        assert n_pos[0] == k and n_tot[0] == n
        assert mean[0] == np.float32(k) / np.float32(n)
        assert abs(float(var[0]) - k * (n - k) / (n * n)) < 1e-7
        if k in (0, n):
            assert var[0] == 0.0          # all-wrong / all-correct: exactly zero


def test_stats_general_rewards_and_ragged_groups():
    rng = np.random.default_rng(0)
    sizes = [3, 0, 7, 1, 16]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = rng.standard_normal(off[-1]).astype(np.float32)
    n_pos, n_tot, mean, var = al.group_stats(r, off)
    for p, s in enumerate(sizes):
        g = r[off[p]:off[p + 1]].astype(np.float64)
        assert n_tot[p] == s
        if s == 0:
            assert mean[p] == 0 and var[p] == 0 and n_pos[p] == 0
            continue
        assert abs(mean[p] - g.mean()) < 1e-6
        assert abs(var[p] - g.var(ddof=0)) < 1e-6          # population: divide by G, not G-1
    assert abs(var[0] - r[:3].astype(np.float64).var(ddof=1)) > 1e-3


def test_filter_truth_table():
    # thresholds of Section 4.2: too easy if > 0.75, too hard if < 0.125,
    # evicted only when every pilot rollout is correct (p_solve = 1)
    keep_k = {4: {1, 2, 3}, 8: set(range(1, 7)), 16: set(range(2, 13)), 32: set(range(4, 25))}
    for n, keep in keep_k.items():
        ph = (np.arange(n + 1, dtype=np.float32) / np.float32(n))
        cls, evict, commit, surplus, counts = al.select_commit(ph, 0.125, 0.75, 1.0)
        assert set(np.nonzero(cls == al.KEEP)[0]) == keep
        assert all(cls[k] == al.HARD for k in range(min(keep)))
        assert all(cls[k] == al.EASY for k in range(max(keep) + 1, n + 1))
        assert list(np.nonzero(evict)[0]) == [n]
        assert list(commit) == sorted(keep) and len(surplus) == 0
        assert list(counts) == [len(keep), 0, n - max(keep), min(keep)]


def test_threshold_edges_inclusive():
    ph = np.array([0.125, 0.75, np.nextafter(np.float32(0.125), np.float32(0)),
                   np.nextafter(np.float32(0.75), np.float32(1))], np.float32)
    cls, evict, *_ = al.select_commit(ph, 0.125, 0.75, 1.0)
    assert list(cls) == [al.KEEP, al.KEEP, al.HARD, al.EASY]
    # eviction is ">=" and independent of the class
    cls, evict, commit, _, _ = al.select_commit(np.array([0.5, 0.75, 0.25], np.float32), 0.125, 0.75, 0.5)
    assert list(evict) == [1, 1, 0] and list(cls) == [al.KEEP] * 3 and list(commit) == [0, 1, 2]


def test_select_brute_force_patterns_and_cap():
    # every keep/skip pattern of P = 10 prompts, with and without a cap
    P = 10
    val = {0: 0.0, 1: 0.5, 2: 1.0}
    rng = np.random.default_rng(0)
    for _ in range(300):
        pat = rng.integers(0, 3, P)
        ph = np.array([val[int(c)] for c in pat], np.float32)
        for b_t in (0, 1, 3, 10, 20):
            cls, evict, commit, surplus, counts = al.select_commit(ph, 0.125, 0.75, 1.0, b_t)
            kept = [q for q in range(P) if pat[q] == 1]
            cap = len(kept) if b_t <= 0 else min(b_t, len(kept))
            assert list(commit) == kept[:cap] and list(surplus) == kept[cap:]
            assert list(np.nonzero(evict)[0]) == [q for q in range(P) if pat[q] == 2]
            assert counts[0] == cap and counts[1] == len(kept) - cap
            assert counts[2] == int((pat == 2).sum()) and counts[3] == int((pat == 0).sum())
    for pat in itertools.product([0, 1], repeat=8):
        ph = np.array([0.5 if c else 0.0 for c in pat], np.float32)
        _, _, commit, _, _ = al.select_commit(ph, 0.125, 0.75, 1.0)
        assert list(commit) == [i for i, c in enumerate(pat) if c]


def test_empty_and_all_kept():
    cls, evict, commit, surplus, counts = al.select_commit(np.zeros(0, np.float32), 0.125, 0.75, 1.0)
    assert len(cls) == 0 and len(commit) == 0 and list(counts) == [0, 0, 0, 0]
    _, _, commit, _, counts = al.select_commit(np.zeros(5, np.float32), 0.125, 0.75, 1.0)
    assert len(commit) == 0 and counts[3] == 5
    _, _, commit, _, _ = al.select_commit(np.full(5, 0.5, np.float32), 0.125, 0.75, 1.0)
    assert list(commit) == [0, 1, 2, 3, 4]


@pytest.mark.parametrize("n", [4, 8, 16, 128])
def test_advantage_binary_closed_form_and_invariants(n):
    for k in range(n + 1):
        r = np.random.default_rng(100 + k).permutation(_binary_group(n, k))
        adv, mu, sigma = al.advantages(r, [0, n], eps=0.0)
        if k in (0, n):
            assert np.all(adv == 0.0) and sigma[0] == 0.0      # zero-variance groups give no signal
            continue
        # A+ = sqrt((n-k)/k), A- = -sqrt(k/(n-k))
        assert np.allclose(adv[r == 1], math.sqrt((n - k) / k), atol=1e-6)
        assert np.allclose(adv[r == 0], -math.sqrt(k / (n - k)), atol=1e-6)
        assert abs(float(adv.astype(np.float64).sum())) < 1e-4          # sum_i A_i = 0 (Section 3.2)
        assert abs(float((adv.astype(np.float64) ** 2).sum()) - n) < 1e-3
        # positive advantage mass S+ = sum|d| / (2 sigma) <= G/2, tight at k = n/2
        s_plus = float(adv[adv > 0].sum())
        d = r.astype(np.float64) - float(mu[0])
        assert abs(s_plus - np.abs(d).sum() / (2 * float(sigma[0]))) < 1e-4
        assert s_plus <= n / 2 + 1e-5
        if 2 * k == n:
            assert abs(s_plus - n / 2) < 1e-5
            assert np.allclose(np.abs(adv), 1.0, atol=1e-7)


def test_advantage_tight_case_g8():
    adv, mu, sigma = al.advantages([1, 0, 1, 0, 0, 1, 1, 0], [0, 8], eps=0.0)
    assert list(adv) == [1, -1, 1, -1, -1, 1, 1, -1] and mu[0] == 0.5 and sigma[0] == 0.5


def test_advantage_eps_and_float_rewards():
    r = np.array([0.2, 0.9, 0.4, 0.1, 1.0, 1.0, 1.0], np.float32)
    off = [0, 4, 7]
    adv, mu, sigma = al.advantages(r, off, eps=1e-6)
    g = r[:4].astype(np.float64)
    assert np.allclose(adv[:4], (g - g.mean()) / (g.std() + 1e-6), atol=1e-6)
    assert np.all(adv[4:] == 0.0) and sigma[1] == 0.0 and mu[1] == 1.0
    # continuous rewards obey the same bound
    assert adv[:4][adv[:4] > 0].sum() <= 2.0 + 1e-6


def test_sampling_cost_matches_paper_tables(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "sampling_cost.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for n, npil, ncom, grpo, pc, dapo in (map(int, r) for r in rows):
        assert npil + ncom == n
        assert al.sampling_cost("grpo", 128, n=n) == grpo
        assert al.sampling_cost("dapo", 128, n=n, s=3) == dapo
        assert al.sampling_cost("pc", 128, s=3, n_pilot=npil, n_commit=ncom) == pc
    assert al.rollouts_generated(64, 4, 29, 4) == 64 * 4 + 29 * 4


def test_rollouts_generated_reproduces_the_printed_per_step_counts(golden_dir):
    # a step whose sampling batch holds b_g = 3 * 128 prompts and whose commit pass keeps exactly b_t = 128
    # generates what the paper prints for Pilot-Commit (Section 4.3; the runtime table; Appendix A.4);
    # and a step that keeps nobody costs the pilot pass alone, b_g * n_pilot
    import os
    for line in open(os.path.join(golden_dir, "sampling_cost.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, n_pilot, n_commit, grpo, pc_count, dapo = map(int, line.split())
        assert al.rollouts_generated(3 * 128, n_pilot, 128, n_commit) == pc_count
        assert al.rollouts_generated(3 * 128, n_pilot, 0, n_commit) == 3 * 128 * n_pilot
        # the same budget spent without a pilot stage: every prompt of the training batch gets n rollouts
        assert al.rollouts_generated(128, n_pilot, 128, n_commit) == grpo


# ---------------------------------------------------------------- rewards that are not binary

def test_variance_filter_reduces_to_the_binary_filter():
    # 0/1 rewards, thresholds p (1 - p) at the paper's p_lower / p_upper, pivot 1/2: the same classes, eviction
    # flags, commit set and counts as the binary filter, for every k at n = 4, 8, 16, 32 (Section 4.2 thresholds;
    # the boundary cases k/n = 0.125 and 0.75 are kept by both)
    for n in (4, 8, 16, 32):
        groups = [np.random.default_rng(k).permutation(_binary_group(n, k)) for k in range(n + 1)]
        off = (np.arange(n + 2) * n).astype(np.int32)
        _, _, mean, var = al.group_stats(np.concatenate(groups), off)
        for b_t in (0, 3):
            want = al.select_commit(mean, 0.125, 0.75, 1.0, b_t)
            got = al.select_commit_variance(mean, var, 0.125 * 0.875, 0.75 * 0.25, 0.5, 1.0, b_t)
            for a, b in zip(want, got):
                assert np.array_equal(a, b)
    # and for random thresholds on either side of 1/2, away from the boundaries
    rng = np.random.default_rng(1)
    for _ in range(50):
        n = int(rng.integers(2, 40))
        lo, hi = rng.uniform(0.01, 0.49), rng.uniform(0.51, 0.99)
        k = np.arange(n + 1)
        if np.min(np.abs(k / n - lo)) < 1e-3 or np.min(np.abs(k / n - hi)) < 1e-3:
            continue
        groups = [_binary_group(n, kk) for kk in k]
        _, _, mean, var = al.group_stats(np.concatenate(groups), (np.arange(n + 2) * n).astype(np.int32))
        want = al.select_commit(mean, lo, hi, 1.0)
        got = al.select_commit_variance(mean, var, lo * (1 - lo), hi * (1 - hi), 0.5, 1.0)
        for a, b in zip(want, got):
            assert np.array_equal(a, b)


def test_variance_filter_multi_valued_rewards_closed_forms():
    # three-valued rewards {0, 1/2, 1}: Var = sum f_v v^2 - mean^2 with f_v the fraction of each value
    groups = {
        "half/half 0 and 1":        ([0, 1, 0, 1],             0.5,   0.25),
        "all one half":             ([.5, .5, .5, .5],         0.5,   0.0),
        "0, 1/2, 1, 1/2":           ([0, .5, 1, .5],           0.5,   0.125),
        "mostly 1/2, one 1":        ([.5, .5, .5, 1],          0.625, 0.046875),
        "mostly 0, one 1/2":        ([0, 0, 0, .5],            0.125, 0.046875),
        "mostly 1, one 0":          ([1, 1, 1, 0],             0.75,  0.1875),
        "all 1":                    ([1, 1, 1, 1],             1.0,   0.0),
    }
    r = np.concatenate([np.asarray(g[0], np.float32) for g in groups.values()])
    off = (np.arange(len(groups) + 1) * 4).astype(np.int32)
    _, _, mean, var = al.group_stats(r, off)
    assert mean.tolist() == [g[1] for g in groups.values()]
    assert var.tolist() == [g[2] for g in groups.values()]
    cls, evict, commit, surplus, counts = al.select_commit_variance(mean, var, 0.04, 0.1, 0.5, 1.0)
    #        0/1 mix   all 1/2 (no spread, mean at the pivot: "approaching")   spread   leaving, too little spread
    assert cls.tolist() == [al.KEEP, al.HARD, al.KEEP, al.EASY, al.KEEP, al.KEEP, al.EASY]
    assert evict.tolist() == [0, 0, 0, 0, 0, 0, 1]
    assert commit.tolist() == [0, 2, 4, 5] and counts.tolist() == [4, 0, 2, 1]
    # a cap keeps the first two in batch order, the rest is surplus
    cls2, _, commit2, surplus2, counts2 = al.select_commit_variance(mean, var, 0.04, 0.1, 0.5, 1.0, b_t=2)
    assert commit2.tolist() == [0, 2] and surplus2.tolist() == [4, 5] and counts2.tolist() == [2, 2, 2, 1]
    assert np.array_equal(cls2, cls)


def test_variance_filter_edges_and_scaling():
    # inclusive thresholds, +-1 ulp
    v = np.float32(0.1)
    below, above = np.nextafter(v, np.float32(0)), np.nextafter(v, np.float32(1))
    mean = np.array([0.3, 0.3, 0.3, 0.7, 0.7, 0.7], np.float32)
    var = np.array([below, v, above, below, v, above], np.float32)
    cls, _, _, _, _ = al.select_commit_variance(mean, var, 0.1, 0.1, 0.5, 2.0)
    assert cls.tolist() == [al.HARD, al.KEEP, al.KEEP, al.EASY, al.KEEP, al.KEEP]
    # the pivot itself counts as "approaching" (<=)
    half = np.float32(0.5)
    cls, _, _, _, _ = al.select_commit_variance([half, np.nextafter(half, np.float32(1))], [0.05, 0.05], 0.04, 0.06, 0.5, 2.0)
    assert cls.tolist() == [al.KEEP, al.EASY]
    # rewards scaled by 4 (exactly representable): variance scales by 16, mean and pivot by 4: same selection
    rng = np.random.default_rng(2)
    r = rng.integers(0, 5, 64 * 8).astype(np.float32) / 4.0
    off = (np.arange(65) * 8).astype(np.int32)
    _, _, m1, v1 = al.group_stats(r, off)
    _, _, m4, v4 = al.group_stats(4.0 * r, off)
    a = al.select_commit_variance(m1, v1, 0.08, 0.11, 0.5, 0.9, 5)
    b = al.select_commit_variance(m4, v4, 16 * 0.08, 16 * 0.11, 2.0, 3.6, 5)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert 0 < a[4][0] and a[4][2] > 0 and a[4][3] > 0          # all three classes occur
    # evict: mean >= mean_solve, independent of the class
    _, evict, _, _, _ = al.select_commit_variance([0.9, 1.0, 1.0], [0.2, 0.0, 0.3], 0.1, 0.1, 0.5, 1.0)
    assert evict.tolist() == [0, 1, 1]
    # empty batch
    out = al.select_commit_variance([], [], 0.1, 0.1, 0.5, 1.0)
    assert len(out[0]) == 0 and out[4].tolist() == [0, 0, 0, 0]
