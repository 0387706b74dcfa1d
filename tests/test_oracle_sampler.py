"""Pins for oracle.sampler: closed forms, monotonicity, distribution."""
import math

import numpy as np
import pytest

from oracle import philox, sampler


def test_two_token_closed_form():
    # token 0 iff u < p0 = 1 / (1 + exp((b - a)/T))
    a, b, T = 0.3, -1.1, 0.7
    p0 = 1.0 / (1.0 + math.exp((b - a) / T))
    for u in np.linspace(0.001, 0.999, 97):
        tok, lp = sampler.sample_token([a, b], T, u)
        assert tok == (0 if u < p0 else 1)
        want_lp = math.log(p0) if tok == 0 else math.log(1 - p0)
        assert abs(lp - want_lp) < 1e-6


def test_one_hot_and_monotone():
    x = np.full(50, -1e4, np.float32)
    x[37] = 0.0
    for u in (1e-7, 0.5, 1 - 1e-7):
        assert sampler.sample_token(x, 1.0, u)[0] == 37
    rng = np.random.default_rng(0)
    logits = rng.standard_normal(300).astype(np.float32)
    us = np.sort(rng.random(200))
    toks = [sampler.sample_token(logits, 1.0, u)[0] for u in us]
    assert all(t1 <= t2 for t1, t2 in zip(toks, toks[1:]))
    # the interval of u mapping to token i is [cdf(i-1), cdf(i))
    p = sampler.softmax_probs(logits)
    cdf = np.cumsum(p)
    for i in (0, 1, 150, 299):
        lo = 0.0 if i == 0 else cdf[i - 1]
        mid = 0.5 * (lo + cdf[i])
        assert sampler.sample_token(logits, 1.0, mid)[0] == i


def test_last_token_when_rounding_leaves_no_crossing():
    # u*Z can equal the total only by rounding; then the last token with
    # non-zero weight is taken, never an index past the end
    x = np.array([0.0, 0.0, -1e9], np.float32)
    tok, _ = sampler.sample_token(x, 1.0, np.nextafter(1.0, 0.0))
    assert tok in (1,)


def test_logprob_is_log_softmax_and_temperature():
    rng = np.random.default_rng(3)
    logits = (3.0 * rng.standard_normal(64)).astype(np.float32)
    for T in (0.5, 1.0, 2.0):
        p = sampler.softmax_probs(logits, T)
        for u in (0.1, 0.6, 0.95):
            tok, lp = sampler.sample_token(logits, T, u)
            assert abs(lp - math.log(p[tok])) < 1e-9


def test_eos_bias_moves_mass_to_eos():
    logits = np.zeros(8, np.float32)
    # bias ln(7) on token 5 makes it as likely as the other seven together
    hits = 0
    n = 4000
    for t in range(n):
        u = philox.sampling_uniform(9, 1, t)
        tok, _ = sampler.sample_token(logits, 1.0, u, eos_id=5, eos_logit_bias=math.log(7.0))
        hits += tok == 5
    assert abs(hits / n - 0.5) < 0.03
    assert sampler.sample_token(logits, 1.0, 0.5, eos_id=-1, eos_logit_bias=100.0)[0] == 4


def test_distribution_chi_square():
    rng = np.random.default_rng(5)
    V, n = 24, 60_000
    logits = rng.standard_normal(V).astype(np.float32)
    p = sampler.softmax_probs(logits)
    counts = np.zeros(V)
    for t in range(n):
        counts[sampler.sample_token(logits, 1.0, philox.sampling_uniform(42, 7, t))[0]] += 1
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 70.0          # 23 dof: mean 23, sd 6.8


# ---------------------------------------------------------------- nucleus (top-p) truncation

def test_top_p_one_is_the_plain_sampler():
    rng = np.random.default_rng(3)
    logits = (2.0 * rng.standard_normal(500)).astype(np.float32)
    for u in rng.random(40):
        assert sampler.sample_token(logits, 0.7, u, top_p=1.0) == sampler.sample_token(logits, 0.7, u)
    assert sampler.nucleus(np.exp(logits.astype(np.float64)), 1.0).all()


def test_top_p_three_token_worked_example():
    # probabilities (0.5, 0.3, 0.2).  top_p = 0.7: 0.5 < 0.7 <= 0.5 + 0.3, so tokens {0, 1} stay and are
    # renormalised to (0.625, 0.375); token 2 is never drawn.  top_p = 0.5: token 0 alone reaches it.
    # top_p = 0.81: all three are needed.
    lg = np.log(np.array([0.5, 0.3, 0.2]))
    for u in np.linspace(0.002, 0.998, 250):
        tok, lp = sampler.sample_token(lg, 1.0, u, top_p=0.7)
        assert tok == (0 if u < 0.625 else 1)
        assert abs(lp - math.log(0.625 if tok == 0 else 0.375)) < 1e-6
        assert sampler.sample_token(lg, 1.0, u, top_p=0.5) == (0, pytest.approx(0.0, abs=1e-6))
        tok3, lp3 = sampler.sample_token(lg, 1.0, u, top_p=0.81)
        assert tok3 == (0 if u < 0.5 else 1 if u < 0.8 else 2)
        assert abs(lp3 - math.log([0.5, 0.3, 0.2][tok3])) < 1e-6
    # the kept tokens need not be a prefix in id order: (0.2, 0.5, 0.3) keeps ids {1, 2}, sampled in id order
    lg2 = np.log(np.array([0.2, 0.5, 0.3]))
    for u in np.linspace(0.002, 0.998, 250):
        assert sampler.sample_token(lg2, 1.0, u, top_p=0.7)[0] == (1 if u < 0.625 else 2)


def test_top_p_ties_keep_the_lower_ids():
    assert sampler.nucleus(np.ones(4), 0.5).tolist() == [True, True, False, False]
    assert sampler.nucleus(np.ones(4), 0.51).tolist() == [True, True, True, False]
    assert sampler.nucleus(np.array([1.0, 4.0, 1.0, 4.0, 1.0]), 0.8).tolist() == [True, True, False, True, False]


def test_top_p_set_is_minimal_and_reaches_the_mass():
    rng = np.random.default_rng(9)
    for trial in range(20):
        w = np.exp(3.0 * rng.standard_normal(400))
        top_p = float(np.float32(rng.uniform(0.05, 0.99)))
        keep = sampler.nucleus(w, top_p)
        mass = w[keep].sum() / w.sum()
        assert mass >= top_p - 1e-12
        assert (w[keep].sum() - w[keep].min()) / w.sum() < top_p + 1e-12        # one token fewer falls short
        assert w[keep].min() >= w[~keep].max()                                  # the heaviest tokens are the kept ones


def test_top_p_distribution_and_temperature():
    # draws at temperature 0.7 with top_p 0.9 follow the softmax at that temperature, truncated and renormalised
    rng = np.random.default_rng(4)
    logits = rng.standard_normal(30).astype(np.float32)
    p = sampler.softmax_probs(logits, 0.7)
    keep = sampler.nucleus(p, 0.9)
    q = np.where(keep, p, 0.0)
    q /= q.sum()
    n = 30000
    counts = np.zeros(30)
    for i in range(n):
        u = philox.sampling_uniform(17, 1000 + i, 0)
        tok, lp = sampler.sample_token(logits, 0.7, u, top_p=0.9)
        counts[tok] += 1
        assert abs(lp - math.log(q[tok])) < 1e-5
    assert counts[~keep].sum() == 0
    chi2 = float((((counts - n * q) ** 2)[keep] / (n * q[keep])).sum())
    assert chi2 < 3.0 * keep.sum()
