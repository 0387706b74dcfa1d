"""Pins of the scoring oracle (Section 3.1: a rollout's probability is the
product of its per-token probabilities)."""
import itertools
import math

import numpy as np
import torch

import workloads
from oracle import decoder, sampler, scoring

TINY = workloads.scaled(workloads.WORKLOADS["C1"], vocab=5, d_model=16, n_q_heads=2, n_kv_heads=1, head_dim=8, d_ff=24,
                        n_layers=2).model


def _weights(std=0.4):
    return workloads.perturb_norm_gains(workloads.make_weights(TINY, 11, std=std), 3)


def test_completions_of_a_prompt_form_a_distribution():
    # chain rule: summed over every possible completion of length 3, the sequence probabilities give exactly 1,
    # and every prefix's next-token probabilities do too
    w = _weights()
    prompt = np.array([3, 1, 4, 1], dtype=np.int64)
    for T in (1.0, 0.7):
        total = 0.0
        for comp in itertools.product(range(TINY.vocab), repeat=3):
            lp = scoring.score(TINY, w, np.concatenate([prompt, comp]), len(prompt), T)
            assert lp.shape == (3,) and (lp < 0).all()
            total += math.exp(lp.sum())
        assert abs(total - 1.0) < 1e-12


def test_matches_the_library_log_softmax_and_the_sampler():
    w = _weights()
    rng = np.random.default_rng(0)
    seq = rng.integers(0, TINY.vocab, 9)
    for T in (1.0, 1.7):
        lp = scoring.score(TINY, w, seq, 4, T)
        logits = decoder.forward_full(TINY, w, seq[:-1], rows=np.arange(3, 8))
        want = torch.log_softmax(torch.from_numpy(logits) / T, dim=-1).numpy()
        for i in range(5):
            assert abs(lp[i] - want[i, seq[4 + i]]) < 1e-12
            # the sampler reports the same number for the token it draws
            for u in (0.1, 0.5, 0.9):
                tok, slp = sampler.sample_token(logits[i], T, u)
                assert abs(slp - scoring.log_softmax_at(logits[i], T, tok)) < 1e-6


def test_closed_forms_and_edges():
    # two equal logits: log(1/2); a dominant logit: ~0 for it, ~ -gap for the others; temperature scales the gap
    assert abs(scoring.log_softmax_at([1.0, 1.0], 1.0, 0) - math.log(0.5)) < 1e-15
    assert abs(scoring.log_softmax_at([0.0, 2.0], 2.0, 0) - (-1.0 - math.log1p(math.exp(-1.0)))) < 1e-15
    assert abs(scoring.log_softmax_at([50.0, 0.0, 0.0], 1.0, 1) - (-50.0 - math.log1p(2 * math.exp(-50.0)))) < 1e-12
    w = _weights()
    seq = np.array([1, 2, 3, 4, 0])
    assert scoring.score(TINY, w, seq, 5).shape == (0,)          # nothing to score
    assert scoring.score(TINY, w, seq, 4).shape == (1,)
    # scoring depends on the prompt: a different first token changes the completion's probabilities
    a = scoring.score(TINY, w, seq, 2)
    b = scoring.score(TINY, w, np.array([0, 2, 3, 4, 0]), 2)
    assert np.abs(a - b).max() > 1e-6
    # and not on what follows a token (causality)
    c = scoring.score(TINY, w, np.array([1, 2, 3, 4, 3]), 2)
    assert np.allclose(a[:2], c[:2], atol=1e-14) and abs(a[2] - c[2]) > 1e-9
