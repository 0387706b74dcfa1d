"""End-to-end checks of oracle.rollout on the tiny workload: its parts are
pinned elsewhere; here the wiring (uids, steps, union groups, counts)."""
import numpy as np

import workloads
from oracle import allocation, decoder, philox, rewards, rollout, sampler

WL = workloads.WORKLOADS["C1"]


def _setup():
    w = workloads.make_weights(WL.model, WL.seed_weights)
    prompts = workloads.make_prompts(WL.n_prompts, WL.prompt_len, WL.model.vocab, WL.seed_prompts)
    uids = workloads.make_prompt_uids(WL.n_prompts)
    return w, prompts, uids


def test_pilot_commit_step_c1_wiring():
    w, prompts, uids = _setup()
    out = rollout.pilot_commit_step(WL, w, prompts, uids, WL.seed_sampler)
    P, T = WL.n_prompts, WL.new_tokens
    assert out["pilot_tokens"].shape == (P, 4, T) and (out["pilot_lens"] == T).all()
    # every token re-derived by brute force: teacher-forced full recompute + the same uniform
    q, j = 3, 2
    seq = np.concatenate([prompts[q], out["pilot_tokens"][q, j]])
    logits = decoder.forward_full(WL.model, w, seq[:-1])
    for t in range(T):
        u = philox.sampling_uniform(WL.seed_sampler, philox.seq_uid(uids[q], j), t)
        tok, _ = sampler.sample_token(logits[WL.prompt_len - 1 + t], WL.temperature, u)
        assert tok == out["pilot_tokens"][q, j, t]
    # rewards follow the rule, stats follow the rewards
    want_r = (out["pilot_tokens"][:, :, -1] % 2 == 0).astype(np.float32)
    assert np.array_equal(out["pilot_rewards"], want_r)
    assert np.array_equal(out["p_hat"], want_r.mean(1).astype(np.float32))
    kept = [q for q in range(P) if 1 <= want_r[q].sum() <= 3]
    assert list(out["commit_idx"]) == kept
    assert out["rollouts"] == P * 4 + len(kept) * 4
    assert out["tokens_generated"] == out["rollouts"] * T
    # commit rollouts use rollout indices n_pilot.. and so differ from the pilot ones
    if kept:
        a, q = 0, kept[0]
        seq = np.concatenate([prompts[q], out["commit_tokens"][a, 1]])
        logits = decoder.forward_full(WL.model, w, seq[:-1])
        u = philox.sampling_uniform(WL.seed_sampler, philox.seq_uid(uids[q], 4 + 1), 5)
        assert sampler.sample_token(logits[WL.prompt_len - 1 + 5], 1.0, u)[0] == out["commit_tokens"][a, 1, 5]
        # advantages over the union group of 8
        g = out["union_rewards"][a].astype(np.float64)
        assert out["union_rewards"].shape[1] == 8
        assert np.array_equal(g[:4], want_r[q])
        if g.std() > 0:
            assert np.allclose(out["advantages"][a], (g - g.mean()) / (g.std() + 1e-6), atol=1e-6)
        assert abs(out["advantages"][a].sum()) < 1e-5


def test_eos_stops_a_rollout():
    w, prompts, uids = _setup()
    # bias an EOS id so that stops happen within 16 tokens
    eos = workloads.make_eos_id(WL.model.vocab, WL.seed_eos)
    toks, lens, lps, _ = rollout.generate_group(WL.model, w, prompts[0], 0, range(6), 16, 1.0, 3,
                                               eos_id=eos, eos_logit_bias=np.log(WL.model.vocab / 4.0))
    assert (lens < 16).any()
    for a in range(6):
        L = lens[a]
        if L < 16:
            assert toks[a, L - 1] == eos and (toks[a, L:] == -1).all()
        assert (toks[a, : L - 1] != eos).all()


def test_class_fractions_beta_bernoulli():
    # Beta(1/2,1/2)-Bernoulli pilot groups: closed-form Beta-Binomial class
    # probabilities for n = 4 (hard k=0, easy k=4, keep otherwise):
    # P(k=0) = P(k=4) = B(1/2, 9/2)/B(1/2, 1/2) = 35/128
    P = 20000
    p_q = workloads.make_success_probs(P, 1)
    u = workloads.make_reward_uniforms(P, 4, 2)
    r = (u < p_q[:, None]).astype(np.float32)
    _, _, p_hat, _ = allocation.group_stats(r.reshape(-1), np.arange(P + 1) * 4)
    cls, evict, commit, _, counts = allocation.select_commit(p_hat, 0.125, 0.75, 1.0)
    assert abs(counts[3] / P - 35 / 128) < 0.012
    assert abs(counts[2] / P - 35 / 128) < 0.012
    assert abs(counts[0] / P - 58 / 128) < 0.012
    assert evict.sum() == counts[2]


def test_reward_rules_worked_examples():
    # each rule on inputs worked by hand from the workload descriptions (none of these repeats the rule's
    # own expression): "1 if the last sampled token id is even"
    for tok, want in ((10, 1.0), (7, 0.0), (0, 1.0), (151935, 0.0), (151934, 1.0)):
        assert rewards.reward("last_even", last_tok=tok) == want
    # "1 if the token id at position -1 mod 7 equals the prompt id mod 7":
    #   15 = 2*7 + 1 and 8 = 7 + 1 agree; 15 against 9 = 7 + 2 does not; 7 and 0 are both multiples of 7;
    #   13 = 7 + 6 against 6; 3 against 10 = 7 + 3; 151935 = 21705*7 + 0 against 14; 100 = 14*7 + 2 against 3
    for tok, uid, want in ((15, 8, 1.0), (15, 9, 0.0), (7, 0, 1.0), (13, 6, 1.0), (3, 10, 1.0), (151935, 14, 1.0),
                           (100, 3, 0.0), (6, 7, 0.0), (1, 7, 0.0), (0, 7, 1.0)):
        assert rewards.reward("last_mod7", last_tok=tok, prompt_uid=uid) == want
    # Bernoulli(p) from a uniform on [0,1): success exactly when the uniform falls below p
    for u, p, want in ((0.25, 0.5, 1.0), (0.5, 0.5, 0.0), (0.75, 0.5, 0.0), (0.0, 0.0, 0.0), (0.0, 1e-9, 1.0),
                       (0.999999, 1.0, 1.0), (0.3, 0.29999, 0.0)):
        assert rewards.reward("bernoulli", p_q=p, u=u) == want
    # success frequency over many uniforms is p
    us = workloads.make_reward_uniforms(1, 40000, 3)[0]
    for p in (0.1, 0.5, 0.83):
        f = np.mean([rewards.reward("bernoulli", p_q=p, u=float(x)) for x in us])
        assert abs(f - p) < 4 * np.sqrt(p * (1 - p) / len(us))
    # the last generated token of a sequence that stopped on EOS is the EOS itself (padding after it is ignored)
    assert rewards.last_token(np.array([5, 9, 4, -1, -1]), 3) == 4
    assert rewards.last_token(np.array([5, 9, 4, 8, 2]), 5) == 2
    assert rewards.last_token(np.array([5]), 1) == 5
    # and score_group applies the rule to exactly that token, per rollout
    toks = np.array([[2, 4, 9, -1], [2, 4, 9, 6]])
    got = rollout.score_group("last_even", toks, np.array([3, 4]), prompt_uid=0)
    assert got.tolist() == [0.0, 1.0]
    got = rollout.score_group("last_mod7", toks, np.array([3, 4]), prompt_uid=9)   # 9 = 7 + 2; 9 mod 7 = 2, 6 mod 7 = 6
    assert got.tolist() == [1.0, 0.0]
