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


def test_graded_reward_worked_examples():
    # residues of the last token and of the prompt uid on the circle mod 7: distance 0, 1, 2, 3 -> 1, 2/3, 1/3, 0
    #   14 vs 0: both residue 0;  15 vs 0: 1 apart;  20 (= 2*7 + 6) vs 0: 1 apart the other way round;
    #   16 vs 0: 2;  17 vs 0: 3;  18 (residue 4) vs 0: 3;  19 (residue 5) vs 0: 2;  3 vs 10 (residue 3): 0
    for tok, uid, want in ((14, 0, 1.0), (15, 0, 2 / 3), (20, 0, 2 / 3), (16, 0, 1 / 3), (17, 0, 0.0), (18, 0, 0.0),
                           (19, 0, 1 / 3), (3, 10, 1.0), (0, 6, 2 / 3), (151935, 13, 2 / 3)):
        got = rewards.reward("graded_mod7", last_tok=tok, prompt_uid=uid)
        assert abs(got - want) < 1e-7, (tok, uid, got, want)
    vals = {rewards.reward("graded_mod7", last_tok=t, prompt_uid=5) for t in range(70)}
    assert len(vals) == 4 and min(vals) == 0.0 and max(vals) == 1.0


def test_step_with_top_p_and_the_variance_filter():
    # the step's wiring with evaluation-style sampling (temperature 0.7, top_p 0.9) and a four-valued reward
    # selected on by the variance filter
    wl = workloads.scaled(WL, temperature=0.7, top_p=0.9, reward="graded_mod7", filter="variance", var_hard=0.02,
                          var_easy=0.05, n_prompts=6, new_tokens=6)
    w, prompts, uids = _setup()
    prompts, uids = prompts[:6], uids[:6]
    out = rollout.pilot_commit_step(wl, w, prompts, uids, 3)
    # a token is always inside the nucleus of its own logits, and is the top-p sampler's choice
    q, j = 2, 1
    seq = np.concatenate([prompts[q], out["pilot_tokens"][q, j]])
    logits = decoder.forward_full(wl.model, w, seq[:-1])
    for t in range(wl.new_tokens):
        lg = logits[wl.prompt_len - 1 + t]
        u = philox.sampling_uniform(3, philox.seq_uid(uids[q], j), t)
        assert sampler.sample_token(lg, 0.7, u, top_p=0.9)[0] == out["pilot_tokens"][q, j, t]
        x = np.asarray(lg, np.float32).astype(np.float64) / 0.7
        assert sampler.nucleus(np.exp(x - x.max()), 0.9)[out["pilot_tokens"][q, j, t]]
    want_r = np.array([[rewards.reward("graded_mod7", last_tok=int(t[-1]), prompt_uid=int(uids[a])) for t in row]
                       for a, row in enumerate(out["pilot_tokens"])], np.float32)
    assert np.array_equal(out["pilot_rewards"], want_r)
    mean, var = want_r.astype(np.float64).mean(1), want_r.astype(np.float64).var(1)
    kept = [a for a in range(6) if (var[a] >= 0.02 - 1e-9 if mean[a] <= 0.5 else var[a] >= 0.05 - 1e-9)]
    assert list(out["commit_idx"]) == kept
    assert out["union_rewards"].shape == (len(kept), 8)
