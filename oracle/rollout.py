"""One Pilot-Commit sampling step, end to end, on the CPU (Algorithm 1 without
the replay buffer): pilot rollouts for every prompt of the batch, pilot
success rates, filter / eviction / commit set, commit rollouts for the kept
prompts, group-relative advantages over pilot U commit.

Test infrastructure.  "parity unpinned" for the token sequences themselves
(no published values exist); every part used here is pinned on its own.
"""
from __future__ import annotations

import numpy as np

from . import allocation, philox, rewards, sampler
from .decoder import CachedDecoder


def generate_group(model, w, prompt, prompt_uid, rollout_indices, new_tokens, temperature, seed,
                   eos_id=-1, eos_logit_bias=0.0, dtype=np.float64, keep_logits=False, top_p=1.0):
    """Sample len(rollout_indices) completions of one prompt (Section 3.1).

    The prompt is run through the model once; every rollout continues from a
    copy of that state.  Token t of a rollout (t = 0 .. new_tokens-1) is drawn
    with the uniform of (seed, sequence uid, step t).  A rollout stops after
    emitting eos_id.  Returns tokens [n, new_tokens] (int32, -1 after the end),
    lengths [n], logprobs [n, new_tokens] (and the logits per step if asked)."""
    base = CachedDecoder(model, w, dtype)
    first_logits = base.extend(prompt)
    n = len(rollout_indices)
    toks = np.full((n, new_tokens), -1, np.int32)
    lps = np.zeros((n, new_tokens), np.float32)
    lens = np.zeros(n, np.int32)
    all_logits = [] if keep_logits else None
    for a, j in enumerate(rollout_indices):
        uid = philox.seq_uid(prompt_uid, j)
        dec = base.clone()
        logits = first_logits
        seq_logits = []
        for t in range(new_tokens):
            if keep_logits:
                seq_logits.append(np.asarray(logits, np.float32))
            u = philox.sampling_uniform(seed, uid, t)
            tok, lp = sampler.sample_token(logits, temperature, u, eos_id, eos_logit_bias, top_p)
            toks[a, t], lps[a, t] = tok, lp
            lens[a] = t + 1
            if tok == eos_id:
                break
            if t + 1 < new_tokens:
                logits = dec.extend([tok])
        if keep_logits:
            all_logits.append(seq_logits)
    return toks, lens, lps, all_logits


def score_group(rule, toks, lens, prompt_uid, p_q=None, reward_u=None):
    out = np.zeros(len(lens), np.float32)
    for a in range(len(lens)):
        out[a] = rewards.reward(rule, last_tok=rewards.last_token(toks[a], lens[a]), prompt_uid=prompt_uid,
                                p_q=p_q, u=None if reward_u is None else reward_u[a])
    return out


def pilot_commit_step(wl, w, prompts, prompt_uids, seed, eos_id=-1, eos_logit_bias=0.0,
                      p_q=None, reward_u=None, dtype=np.float64):
    """wl: a workload description (n_pilot, n_commit, new_tokens, temperature,
    reward, thresholds, b_t, model).  prompts: [P, Lp] or list of arrays.
    Returns a dict with everything the step produces."""
    P = len(prompts)
    npil, ncom, T = wl.n_pilot, wl.n_commit, wl.new_tokens
    top_p = getattr(wl, "top_p", 1.0)
    pilot_tok = np.full((P, npil, T), -1, np.int32)
    pilot_len = np.zeros((P, npil), np.int32)
    pilot_r = np.zeros((P, npil), np.float32)
    for q in range(P):
        t, l, _, _ = generate_group(wl.model, w, prompts[q], int(prompt_uids[q]), range(npil), T,
                                    wl.temperature, seed, eos_id, eos_logit_bias, dtype, top_p=top_p)
        pilot_tok[q], pilot_len[q] = t, l
        pilot_r[q] = score_group(wl.reward, t, l, int(prompt_uids[q]),
                                 None if p_q is None else p_q[q],
                                 None if reward_u is None else reward_u[q, :npil])
    off = np.arange(P + 1, dtype=np.int32) * npil
    n_pos, n_tot, p_hat, var = allocation.group_stats(pilot_r.reshape(-1), off)
    if getattr(wl, "filter", "binary") == "variance":
        cls, evict, commit_idx, surplus_idx, counts = allocation.select_commit_variance(
            p_hat, var, wl.var_hard, wl.var_easy, wl.mean_pivot, wl.p_solve, wl.b_t)
    else:
        cls, evict, commit_idx, surplus_idx, counts = allocation.select_commit(
            p_hat, wl.p_lower, wl.p_upper, wl.p_solve, wl.b_t)
    K = len(commit_idx)
    commit_tok = np.full((K, ncom, T), -1, np.int32)
    commit_len = np.zeros((K, ncom), np.int32)
    commit_r = np.zeros((K, ncom), np.float32)
    for a, q in enumerate(commit_idx):
        t, l, _, _ = generate_group(wl.model, w, prompts[q], int(prompt_uids[q]), range(npil, npil + ncom), T,
                                    wl.temperature, seed, eos_id, eos_logit_bias, dtype, top_p=top_p)
        commit_tok[a], commit_len[a] = t, l
        commit_r[a] = score_group(wl.reward, t, l, int(prompt_uids[q]),
                                  None if p_q is None else p_q[q],
                                  None if reward_u is None else reward_u[q, npil:npil + ncom])
    union_r = np.concatenate([pilot_r[commit_idx], commit_r], axis=1) if K else np.zeros((0, npil + ncom), np.float32)
    uoff = np.arange(K + 1, dtype=np.int32) * (npil + ncom)
    adv, mu, sigma = allocation.advantages(union_r.reshape(-1), uoff)
    return dict(pilot_tokens=pilot_tok, pilot_lens=pilot_len, pilot_rewards=pilot_r,
                n_pos=n_pos, n_tot=n_tot, p_hat=p_hat, var=var, cls=cls, evict=evict,
                commit_idx=commit_idx, surplus_idx=surplus_idx, counts=counts,
                commit_tokens=commit_tok, commit_lens=commit_len, commit_rewards=commit_r,
                union_rewards=union_r, advantages=adv.reshape(K, npil + ncom), mu=mu, sigma=sigma,
                rollouts=allocation.rollouts_generated(P, npil, K, ncom),
                tokens_generated=int(pilot_len.sum() + commit_len.sum()))
