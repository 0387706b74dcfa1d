"""Pilot-Commit allocation rules, written out from their definitions.

Test infrastructure: reference for pc_group_stats / pc_select_commit /
pc_advantages.

  group_stats     Eq. 3 (mean and population variance of a group's rewards);
                  Section 3.3: pilot success rate p_hat = (1/n) sum r_j, with
                  Var[r|q] = p(1-p) for binary rewards
  select_commit   Section 3.3 filter B' = {q : p_lower <= p_hat <= p_upper};
                  Algorithm 1 eviction {q : p_hat >= p_solve}; Section 3.3
                  cap of b_t on the committed prompts, surplus survivors kept
                  aside (for the replay buffer)
  select_commit_variance
                  the same filter on the group variance itself, for rewards
                  that are not binary (Introduction, Section 3.3, Section 7:
                  the paper names the extension, the rule is this implementation's
                  reading)
  advantages      Section 3.1: A_i = (r_i - mu) / sigma over the union of a
                  kept prompt's pilot and commit rollouts (Section 3.3,
                  "Training")
  sampling_cost   Section 4.3 per-step rollout counts

Threshold comparisons are taken in fp32 on the fp32 value of p_hat (the
library takes the same decisions in the same precision).
"""
from __future__ import annotations

import numpy as np

HARD, KEEP, EASY = 0, 1, 2


def group_stats(rewards, group_off):
    """rewards: [N] float; group_off: [P+1] offsets.  Per group: number of
    non-zero rewards, group size, mean (fp32) and population variance (fp32,
    divide by the group size, Eq. 3).  Sums are float64 in index order, two
    passes; an empty group gets mean = var = 0."""
    r = np.asarray(rewards, dtype=np.float32).astype(np.float64)
    off = np.asarray(group_off, dtype=np.int64)
    P = len(off) - 1
    n_pos = np.zeros(P, np.int32)
    n_tot = np.zeros(P, np.int32)
    mean = np.zeros(P, np.float32)
    var = np.zeros(P, np.float32)
    for p in range(P):
        g = r[off[p]:off[p + 1]]
        n = len(g)
        n_tot[p] = n
        n_pos[p] = int(np.count_nonzero(g))
        if n == 0:
            continue
        s = 0.0
        for x in g:
            s += x
        mu = s / n
        ss = 0.0
        for x in g:
            ss += (x - mu) * (x - mu)
        mean[p] = np.float32(mu)
        var[p] = np.float32(ss / n)
    return n_pos, n_tot, mean, var


def select_commit(p_hat, p_lower, p_upper, p_solve, b_t=0):
    """p_hat: [P] fp32 pilot success rates, in batch order.

    cls[q]   = EASY if p_hat > p_upper, HARD if p_hat < p_lower, else KEEP
    evict[q] = p_hat >= p_solve        (independent of cls)
    commit   = the first min(#KEEP, b_t) kept indices, ascending (b_t <= 0:
               no cap); surplus = the remaining kept indices, ascending.
    Returns (cls u8, evict u8, commit_idx i32, surplus_idx i32,
             counts i32[4] = n_commit, n_surplus, n_easy, n_hard)."""
    ph = np.asarray(p_hat, dtype=np.float32)
    lo, hi, so = np.float32(p_lower), np.float32(p_upper), np.float32(p_solve)
    P = len(ph)
    cls = np.empty(P, np.uint8)
    evict = np.zeros(P, np.uint8)
    commit, surplus = [], []
    for q in range(P):
        if ph[q] > hi:
            cls[q] = EASY
        elif ph[q] < lo:
            cls[q] = HARD
        else:
            cls[q] = KEEP
            if b_t <= 0 or len(commit) < b_t:
                commit.append(q)
            else:
                surplus.append(q)
        if ph[q] >= so:
            evict[q] = 1
    counts = np.array([len(commit), len(surplus), int(np.sum(cls == EASY)), int(np.sum(cls == HARD))], np.int32)
    return cls, evict, np.asarray(commit, np.int32), np.asarray(surplus, np.int32), counts


def select_commit_variance(mean, var, var_hard, var_easy, mean_pivot, mean_solve, b_t=0):
    """Pilot filter for rewards that are not binary, on the pilot group's mean
    and population variance (fp32, as group_stats returns them).

    The paper defines the filter for binary rewards only and says that it
    extends to any scalar reward, with the variance as the measure of a
    prompt's informativeness (Introduction; Section 3.3; Section 7).  The
    reading taken here keeps the two things Section 3.3 argues for -- select on
    the variance, and be more lenient with prompts that still approach the
    high-variance regime than with prompts that have passed it:

      keep[q]  = var >= var_hard   if mean <= mean_pivot   (approaching)
                 var >= var_easy   if mean >  mean_pivot   (leaving)
      cls[q]   = KEEP if kept, else HARD if mean <= mean_pivot, else EASY
      evict[q] = mean >= mean_solve
      commit / surplus: as in select_commit.

    With 0/1 rewards, mean_pivot = 1/2, var_hard = p_lower (1 - p_lower) and
    var_easy = p_upper (1 - p_upper) (p_lower <= 1/2 <= p_upper) this is the
    binary filter p_lower <= p_hat <= p_upper, since p (1 - p) rises up to 1/2
    and falls beyond it.  All comparisons in fp32."""
    mu = np.asarray(mean, dtype=np.float32)
    vr = np.asarray(var, dtype=np.float32)
    vh, ve = np.float32(var_hard), np.float32(var_easy)
    pv, so = np.float32(mean_pivot), np.float32(mean_solve)
    P = len(mu)
    cls = np.empty(P, np.uint8)
    evict = np.zeros(P, np.uint8)
    commit, surplus = [], []
    for q in range(P):
        approaching = mu[q] <= pv
        kept = (vr[q] >= vh) if approaching else (vr[q] >= ve)
        if kept:
            cls[q] = KEEP
            if b_t <= 0 or len(commit) < b_t:
                commit.append(q)
            else:
                surplus.append(q)
        else:
            cls[q] = HARD if approaching else EASY
        if mu[q] >= so:
            evict[q] = 1
    counts = np.array([len(commit), len(surplus), int(np.sum(cls == EASY)), int(np.sum(cls == HARD))], np.int32)
    return cls, evict, np.asarray(commit, np.int32), np.asarray(surplus, np.int32), counts


def advantages(rewards, group_off, eps=1e-6):
    """A_i = (r_i - mu) / (sigma + eps) per group, sigma the population
    standard deviation (Eq. 3).  With sigma = 0 every r_i - mu is 0 and the
    advantage is defined as exactly 0 (also when eps = 0).
    eps is taken at its fp32 value (the library's argument type).
    Returns (adv fp32 [N], mu fp32 [P], sigma fp32 [P]); float64 inside."""
    r = np.asarray(rewards, dtype=np.float32).astype(np.float64)
    off = np.asarray(group_off, dtype=np.int64)
    P = len(off) - 1
    adv = np.zeros(len(r), np.float32)
    mu_o = np.zeros(P, np.float32)
    sg_o = np.zeros(P, np.float32)
    for p in range(P):
        g = r[off[p]:off[p + 1]]
        n = len(g)
        if n == 0:
            continue
        s = 0.0
        for x in g:
            s += x
        mu = s / n
        ss = 0.0
        for x in g:
            ss += (x - mu) * (x - mu)
        sigma = np.sqrt(ss / n)
        mu_o[p], sg_o[p] = np.float32(mu), np.float32(sigma)
        for i, x in enumerate(g):
            d = x - mu
            adv[off[p] + i] = np.float32(0.0 if d == 0.0 else d / (sigma + float(np.float32(eps))))
    return adv, mu_o, sg_o


def sampling_cost(method, b_t, n=None, s=3, n_pilot=None, n_commit=None):
    """Rollouts sampled per training step (Section 4.3): GRPO b_t*n; DAPO
    b_g*n; Pilot-Commit b_g*n_pilot + b_t*n_commit, with b_g = s*b_t."""
    b_g = s * b_t
    if method == "grpo":
        return b_t * n
    if method == "dapo":
        return b_g * n
    if method == "pc":
        return b_g * n_pilot + b_t * n_commit
    raise ValueError(method)


def rollouts_generated(n_prompts, n_pilot, n_kept, n_commit):
    """Rollouts one pilot + commit step actually generates."""
    return n_prompts * n_pilot + n_kept * n_commit
