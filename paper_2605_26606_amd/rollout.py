"""Host driver of one Pilot-Commit sampling step (Algorithm 1 without the
replay buffer): shared-prefix prefill, pilot rollouts, per-prompt statistics,
filter / commit set, commit rollouts on the kept prompts only, advantages over
pilot U commit.  Every step of the path runs in the library's kernels; this
file only sequences pc_* calls and holds device buffers.  The synthetic reward
rules (the stand-in for the paper's verifier, Section 3.3 R(q,o)) are applied
here with elementwise tensor ops, as a caller would apply its own verifier.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _seq_uids(prompt_uids: np.ndarray, rollout_indices) -> np.ndarray:
    """uid = prompt uid * 2^16 + rollout index, prompt-major."""
    r = np.asarray(list(rollout_indices), dtype=np.int64)
    return (np.asarray(prompt_uids, dtype=np.int64)[:, None] * 65536 + r[None, :]).reshape(-1)


def plan_waves(ctx: B.Context, handles: np.ndarray, new_tokens: int, free_slots_reserve: int = 0):
    """Cuts the sequences (one per entry of `handles`, rollouts of a prompt next to each other) into consecutive
    waves that each fit the free KV blocks, the free slots and the activation buffers of the context; a prompt's
    rollouts stay in one wave.  -> list of (begin, end).  Raises if a single prompt's group does not fit."""
    n = len(handles)
    if n == 0:
        return []
    need = B.pc_fork_need(ctx, handles, new_tokens)
    free_blocks, _ = B.pc_kv_blocks(ctx)
    max_rows = min(ctx.max_batch_rows, B.pc_slots(ctx)[0] - free_slots_reserve)   # a sequence takes a slot
    bounds = [0]
    for i in range(1, n + 1):
        if i == n or handles[i] != handles[i - 1]:
            bounds.append(i)
    waves, b, blocks, rows = [], 0, 0, 0
    for g0, g1 in zip(bounds[:-1], bounds[1:]):
        gb, gr = int(need[g0:g1].sum()), g1 - g0
        if gb > free_blocks or gr > max_rows:
            raise B.PcError(-2, "one prompt's %d rollouts need %d KV blocks / %d rows; the pool has %d free, a decode "
                                "step holds %d rows" % (gr, gb, gr, free_blocks, max_rows))
        if blocks + gb > free_blocks or rows + gr > max_rows:
            waves.append((b, g0))
            b, blocks, rows = g0, 0, 0
        blocks += gb
        rows += gr
    waves.append((b, n))
    return waves


def generate(ctx: B.Context, handles: np.ndarray, logit_rows: np.ndarray, first_logits: torch.Tensor,
             seq_uids: np.ndarray, new_tokens: int, temperature: float, seed: int, eos_id: int = -1,
             eos_logit_bias: float = 0.0, stream=None, **kw):
    """generate_wave over as many waves as the KV pool makes necessary (Section 3.4: on one GPU the pool is shared
    by everything that decodes): when the sequences' reserved blocks do not all fit, the pass is cut into
    consecutive waves, each decoded to the end and released before the next is forked.  A sequence's tokens depend
    on its uid and step only, never on the wave it ran in.  Same arguments and result as generate_wave; logits can
    only be kept (keep_logits_rows) when the pass fits one wave."""
    handles = np.ascontiguousarray(handles, dtype=np.int32)
    waves = plan_waves(ctx, handles, int(new_tokens))
    if len(waves) <= 1:
        return generate_wave(ctx, handles, logit_rows, first_logits, seq_uids, new_tokens, temperature, seed, eos_id,
                             eos_logit_bias, stream, **kw)
    if kw.get("keep_logits_rows") is not None:
        raise ValueError("logits can only be kept when the pass fits one wave (%d needed)" % len(waves))
    outs = []
    for b, e in waves:
        outs.append(generate_wave(ctx, handles[b:e], np.asarray(logit_rows)[b:e], first_logits, np.asarray(seq_uids)[b:e],
                                  new_tokens, temperature, seed, eos_id, eos_logit_bias, stream, **kw))
    out = dict(tokens=torch.cat([o["tokens"] for o in outs]), lengths=torch.cat([o["lengths"] for o in outs]),
               steps_run=sum(o["steps_run"] for o in outs), rows_decoded=sum(o["rows_decoded"] for o in outs),
               logits=[], logits_rows=[], logits_steps=[], waves=len(waves))
    if "logprobs" in outs[0]:
        out["logprobs"] = torch.cat([o["logprobs"] for o in outs])
    return out


def generate_wave(ctx: B.Context, handles: np.ndarray, logit_rows: np.ndarray, first_logits: torch.Tensor,
             seq_uids: np.ndarray, new_tokens: int, temperature: float, seed: int, eos_id: int = -1,
             eos_logit_bias: float = 0.0, stream=None, keep_logits_rows: Optional[np.ndarray] = None,
             poll_every: int = 64, time_class: int = -1, time_every: int = 0, timed_steps: Optional[list] = None,
             compact: bool = True, keep_logprobs: bool = False, top_p: float = 1.0,
             keep_logits_steps: Optional[Sequence[int]] = None):
    """Samples one completion per entry of `handles` (prompt handles, one per
    sequence).  Token 0 comes from the prompt's prefill logits
    (first_logits[logit_rows[i]]); tokens 1.. from decode steps.

    With an EOS id the finished flags are read back every `poll_every` steps;
    when enough sequences have stopped (`compact`), they are released and the
    decode batch shrinks to the live ones (ragged stop), and the pass ends as
    soon as none is left.

    keep_logprobs: also return logprobs [n, T] fp32, the log-probability of
    every sampled token under the sampling distribution (the pi_theta_old of
    Eq. 2; 0 after a sequence's end).

    Returns dict(tokens [n, T] int32 device (eos_id-padded after the end when
    EOS is on), lengths [n] int32 device, steps_run, rows_decoded (sum of the
    batch sizes of the decode steps), logits / logits_rows (optional: per step
    -- or only for the steps in keep_logits_steps, then with logits_steps naming
    them -- the logits of the requested rows that were still in the batch, and
    which rows those are; for parity tests))."""
    dev = first_logits.device
    n = len(handles)
    V = ctx.vocab
    T = int(new_tokens)
    hist = torch.full((T, max(n, 1)), eos_id if eos_id >= 0 else 0, dtype=torch.int32, device=dev)
    out = dict(tokens=hist[:, :n].t().contiguous(), lengths=torch.zeros(n, dtype=torch.int32, device=dev),
               steps_run=0, rows_decoded=0, logits=[], logits_rows=[])
    if n == 0 or T == 0:
        return out
    seqs = B.pc_fork(ctx, handles, T, stream)
    uid_d = torch.from_numpy(np.ascontiguousarray(seq_uids, dtype=np.int64)).to(dev)
    rows_d = torch.from_numpy(np.ascontiguousarray(logit_rows, dtype=np.int32)).to(dev)
    cur = torch.zeros(n, dtype=torch.int32, device=dev)
    logits = torch.empty((n, V), dtype=torch.float32, device=dev)
    finished = torch.zeros(n, dtype=torch.uint8, device=dev) if eos_id >= 0 else None
    keep = None if keep_logits_rows is None else torch.as_tensor(keep_logits_rows, dtype=torch.long, device=dev)
    keep_mask = None
    if keep is not None:
        keep_mask = torch.zeros(n, dtype=torch.bool, device=dev)
        keep_mask[keep] = True
    active = None                      # original index of each batch row (int32, device); None = identity
    lp_hist = torch.zeros((T, n), dtype=torch.float32, device=dev) if keep_logprobs else None
    # the sampler itself files every token (and its log-probability) under [step][original index]: no copy
    # kernel per step, also after the batch has shrunk
    B.pc_sample(first_logits, rows_d, n, V, temperature, seed, uid_d, None, 0, eos_id, eos_logit_bias, cur, None,
                finished, stream, top_p=top_p, hist_tokens=hist[0], hist_logprob=None if lp_hist is None else lp_hist[0])
    keep_steps = None if keep_logits_steps is None else set(int(x) for x in keep_logits_steps)
    out["logits_steps"] = []
    if keep is not None and (keep_steps is None or 0 in keep_steps):
        out["logits"].append(first_logits[rows_d.long()[keep]].clone())
        out["logits_rows"].append(keep.clone())
        out["logits_steps"].append(0)
    steps, rows_decoded = 1, 0
    for t in range(1, T):
        if finished is not None and t % poll_every == 0:
            fin = finished.cpu().numpy().astype(bool)          # the pass's only periodic read-back
            if fin.all():
                break
            if compact and fin.sum() >= max(1, len(fin) // 16):
                alive = np.nonzero(~fin)[0]
                B.pc_release(ctx, seqs[fin], 0)
                seqs = np.ascontiguousarray(seqs[alive])
                alive_d = torch.from_numpy(alive).to(dev)
                active = alive_d.to(torch.int32) if active is None else active[alive_d].contiguous()
                cur = cur[alive_d].contiguous()
                uid_d = uid_d[alive_d].contiguous()
                finished = finished[alive_d].contiguous()
                logits = logits[:len(alive)]
        m = len(seqs)
        if time_every > 0 and t % time_every == time_every // 2:
            # this step runs eagerly with HIP events around every launch of one kernel class
            B.pc_set_option(ctx, B.PC_OPT_TIME_NEXT_STEP, time_class)
            if timed_steps is not None:
                timed_steps.append((t, m))
        B.pc_decode_step(ctx, seqs, cur, logits, stream)
        rows_decoded += m
        if keep is not None and (keep_steps is None or t in keep_steps):
            out["logits_steps"].append(t)
            if active is None:
                out["logits"].append(logits[keep].clone())
                out["logits_rows"].append(keep.clone())
            else:
                act_l = active.long()
                sel = keep_mask[act_l]
                out["logits"].append(logits[sel].clone())
                out["logits_rows"].append(act_l[sel].clone())
        B.pc_sample(logits, None, m, V, temperature, seed, uid_d, None, t, eos_id, eos_logit_bias, cur, None,
                    finished, stream, top_p=top_p, hist_tokens=hist[t],
                    hist_logprob=None if lp_hist is None else lp_hist[t], hist_index=active)
        steps += 1
    B.pc_release(ctx, seqs, 0)
    toks = hist[:, :n].t().contiguous()
    if eos_id >= 0:
        is_eos = (toks == eos_id)
        first = torch.where(is_eos.any(1), is_eos.float().argmax(1).to(torch.int32) + 1,
                            torch.full((n,), T, dtype=torch.int32, device=dev))
        lengths = first.to(torch.int32)
    else:
        lengths = torch.full((n,), T, dtype=torch.int32, device=dev)
    out.update(tokens=toks, lengths=lengths, steps_run=steps, rows_decoded=rows_decoded)
    if keep_logprobs:
        out["logprobs"] = lp_hist.t().contiguous()
    return out


def synthetic_rewards(rule: str, tokens: torch.Tensor, lengths: torch.Tensor, prompt_uid_per_seq: torch.Tensor,
                      p_q_per_seq: Optional[torch.Tensor] = None, reward_u: Optional[torch.Tensor] = None):
    """Binary reward per sequence from its last generated token (the EOS
    itself when the sequence stopped on it)."""
    last = tokens.gather(1, (lengths.long() - 1).clamp(min=0)[:, None])[:, 0].long()
    if rule == "last_even":
        r = (last % 2 == 0)
    elif rule == "last_mod7":
        r = (last % 7 == prompt_uid_per_seq.long() % 7)
    elif rule == "bernoulli":
        r = reward_u < p_q_per_seq
    elif rule == "graded_mod7":
        d = (last - prompt_uid_per_seq.long()) % 7
        d = torch.minimum(d, 7 - d)
        return (3 - d).to(torch.float32) / 3.0
    else:
        raise ValueError(rule)
    return r.to(torch.float32)


def pilot_commit_step(ctx: B.Context, wl, prompt_tokens: torch.Tensor, cu_lens: np.ndarray, prompt_uids: np.ndarray,
                      seed: int, eos_id: int = -1, eos_logit_bias: float = 0.0, p_q: Optional[np.ndarray] = None,
                      reward_u: Optional[np.ndarray] = None, stream=None, eps: float = 1e-6, time_class: int = -1,
                      time_every: int = 0, timed_steps: Optional[list] = None, timings: Optional[dict] = None,
                      log=None):
    """One pilot + commit step for the batch of prompts.  Returns a dict of
    device tensors / host counts mirroring the quantities of Algorithm 1.
    `timings` (optional dict) receives prefill_ms / pilot_ms / commit_ms from
    events on the current stream.  `log` (optional callable) is told when a
    phase has been handed to the GPU and when the selection is known."""
    log = log or (lambda msg: None)
    dev = prompt_tokens.device
    P = len(cu_lens) - 1
    V = ctx.vocab
    npil, ncom, T = wl.n_pilot, wl.n_commit, wl.new_tokens
    uids = np.asarray(prompt_uids, dtype=np.int64)
    last_logits = torch.empty((P, V), dtype=torch.float32, device=dev)
    marks = []

    def mark():
        if timings is not None:
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            marks.append(e)

    mark()
    handles = B.pc_prefill_shared(ctx, prompt_tokens, cu_lens, last_logits, stream)
    mark()
    log("prefill of %d prompts enqueued" % P)
    uid_d = torch.from_numpy(uids).to(dev)
    pq_d = None if p_q is None else torch.from_numpy(np.asarray(p_q, np.float32)).to(dev)
    ru_d = None if reward_u is None else torch.from_numpy(np.asarray(reward_u, np.float32)).to(dev)

    # ---- pilot pass: n_pilot rollouts for every prompt
    rows = np.repeat(np.arange(P, dtype=np.int32), npil)
    tkw = dict(time_class=time_class, time_every=time_every)
    ts_p = [] if timed_steps is not None else None
    ts_c = [] if timed_steps is not None else None
    top_p = float(getattr(wl, "top_p", 1.0))
    g = generate(ctx, handles[rows], rows, last_logits, _seq_uids(uids, range(npil)), T, wl.temperature, seed,
                 eos_id, eos_logit_bias, stream, timed_steps=ts_p, top_p=top_p, **tkw)
    mark()
    rows_d = torch.from_numpy(rows).to(dev).long()
    pilot_r = synthetic_rewards(wl.reward, g["tokens"], g["lengths"], uid_d[rows_d],
                                None if pq_d is None else pq_d[rows_d],
                                None if ru_d is None else ru_d[:, :npil].reshape(-1))
    off = torch.arange(P + 1, dtype=torch.int32, device=dev) * npil
    n_pos = torch.empty(P, dtype=torch.int32, device=dev)
    n_tot = torch.empty(P, dtype=torch.int32, device=dev)
    p_hat = torch.empty(P, dtype=torch.float32, device=dev)
    var = torch.empty(P, dtype=torch.float32, device=dev)
    B.pc_group_stats(pilot_r, off, n_pos, n_tot, p_hat, var, stream)
    cls = torch.empty(P, dtype=torch.uint8, device=dev)
    evict = torch.empty(P, dtype=torch.uint8, device=dev)
    commit_idx = torch.empty(P, dtype=torch.int32, device=dev)
    surplus_idx = torch.empty(P, dtype=torch.int32, device=dev)
    counts = torch.empty(4, dtype=torch.int32, device=dev)
    if getattr(wl, "filter", "binary") == "variance":
        B.pc_select_commit_var(p_hat, var, P, wl.var_hard, wl.var_easy, wl.mean_pivot, wl.p_solve, wl.b_t, cls, evict,
                               commit_idx, surplus_idx, counts, stream)
    else:
        B.pc_select_commit(p_hat, P, wl.p_lower, wl.p_upper, wl.p_solve, wl.b_t, cls, evict, commit_idx, surplus_idx,
                           counts, stream)
    counts_h = counts.cpu().numpy()            # the one read-back the method needs: the commit pass's size
    K = int(counts_h[0])
    kept = commit_idx[:K].cpu().numpy()
    log("pilot pass done (%d sequences x %d tokens); %d of %d prompts kept" % (P * npil, T, K, P))

    # ---- commit pass: n_commit more rollouts for the kept prompts only; prefix KV is reused
    mark()
    crow = np.repeat(kept.astype(np.int32), ncom)
    gc = generate(ctx, handles[crow], crow, last_logits, _seq_uids(uids[kept], range(npil, npil + ncom)), T,
                  wl.temperature, seed, eos_id, eos_logit_bias, stream, timed_steps=ts_c, top_p=top_p)   # timing: pilot pass only
    if timed_steps is not None:
        # (pass, step, sequences, prompts whose prefix those sequences share)
        timed_steps.extend(("pilot", t, n, P) for t, n in ts_p)
        timed_steps.extend(("commit", t, n, K) for t, n in ts_c)
    mark()
    crow_d = torch.from_numpy(crow).to(dev).long()
    commit_r = synthetic_rewards(wl.reward, gc["tokens"], gc["lengths"], uid_d[crow_d],
                                 None if pq_d is None else pq_d[crow_d],
                                 None if ru_d is None else ru_d[torch.from_numpy(kept).to(dev).long(), npil:npil + ncom]
                                 .reshape(-1)) if K else torch.zeros(0, dtype=torch.float32, device=dev)
    B.pc_release(ctx, handles, 1)

    # ---- advantages over the union group of every kept prompt
    kept_d = torch.from_numpy(kept).to(dev).long()
    union_r = torch.cat([pilot_r.view(P, npil)[kept_d], commit_r.view(K, ncom)], dim=1).contiguous()
    uoff = torch.arange(K + 1, dtype=torch.int32, device=dev) * (npil + ncom)
    adv = torch.zeros(K * (npil + ncom), dtype=torch.float32, device=dev)
    mu = torch.zeros(max(K, 1), dtype=torch.float32, device=dev)
    sigma = torch.zeros(max(K, 1), dtype=torch.float32, device=dev)
    if K:
        B.pc_advantages(union_r.view(-1), uoff, eps, adv, mu, sigma, stream)
    n_tok = int(g["lengths"].sum().item()) + (int(gc["lengths"].sum().item()) if K else 0)
    log("commit pass done (%d sequences)" % (K * ncom))
    if timings is not None:
        torch.cuda.current_stream().synchronize()
        timings.update(prefill_ms=marks[0].elapsed_time(marks[1]), pilot_ms=marks[1].elapsed_time(marks[2]),
                       commit_ms=marks[3].elapsed_time(marks[4]))
    return dict(pilot_tokens=g["tokens"].view(P, npil, T), pilot_lens=g["lengths"].view(P, npil),
                pilot_rewards=pilot_r.view(P, npil), n_pos=n_pos, n_tot=n_tot, p_hat=p_hat, var=var, cls=cls,
                evict=evict, commit_idx=kept, surplus_idx=surplus_idx[:int(counts_h[1])].cpu().numpy(),
                counts=counts_h, commit_tokens=gc["tokens"].view(K, ncom, T), commit_lens=gc["lengths"].view(K, ncom),
                commit_rewards=commit_r.view(K, ncom), union_rewards=union_r, advantages=adv.view(K, npil + ncom),
                mu=mu[:K], sigma=sigma[:K], rollouts=P * npil + K * ncom, tokens_generated=n_tok,
                decode_steps=g["steps_run"] + gc["steps_run"])


class BoundPipeline:
    """Pilot/commit binding (Section 3.4) on one GPU: the commit rollouts of the
    prompts selected at step t-1 and the pilot rollouts of the sampling batch
    of step t are generated in ONE decode batch, so the commit pass, which on
    its own is too small to amortise the weight stream, rides along with the
    pilot pass.  Selection between the steps goes through the library's
    scheduler (replay buffer, cap b_t, maximum delay d, eviction).  The prefix
    KV and the last-row logits of a kept prompt stay alive until its commit
    pass has run; everything else is released as soon as it is decided.

    The policy (weights) is the same for every step here, so binding changes
    the schedule, not the results: every sequence gets the tokens it would get
    in an unbound step (same uid, same Philox stream, same logits up to the
    kernels' batch-size-dependent summation order)."""

    def __init__(self, ctx: B.Context, wl, seed: int, eos_id: int = -1, eos_logit_bias: float = 0.0,
                 max_delay: int = 0, b_t: Optional[int] = None, eps: float = 1e-6):
        self.ctx, self.wl, self.seed, self.eos_id, self.eos_bias, self.eps = ctx, wl, seed, eos_id, eos_logit_bias, eps
        cap = b_t if b_t is not None else wl.b_t
        self.sched = B.Scheduler(wl.p_lower, wl.p_upper, wl.p_solve, cap if cap and cap > 0 else (1 << 30) - 1,
                                 max_delay)
        self.entries = {}          # tag -> dict(handle, uid, logits [V] device, pilot_r [n_pilot] device, tokens)
        self.pending = []          # tags selected for the commit pass of the next step
        self.next_tag = 0
        self.step_no = 0

    def close(self):
        for e in self.entries.values():
            B.pc_release(self.ctx, np.array([e["handle"]], np.int32), 1)
        self.entries.clear()
        self.pending = []
        self.sched.close()

    def step(self, prompt_tokens: Optional[torch.Tensor], cu_lens: Optional[np.ndarray],
             prompt_uids: Optional[np.ndarray], p_q: Optional[np.ndarray] = None,
             reward_u: Optional[np.ndarray] = None, stream=None):
        """Runs the pilot pass of this sampling batch (None: no new batch, drain
        only) together with the commit pass of the prompts selected at the
        previous step.  Returns a dict: pilot_* of this batch, commit_* /
        advantages of the prompts whose commit pass just ran."""
        ctx, wl = self.ctx, self.wl
        npil, ncom, T, V = wl.n_pilot, wl.n_commit, wl.new_tokens, ctx.vocab
        P = 0 if cu_lens is None else len(cu_lens) - 1
        com = [self.entries[t] for t in self.pending]
        K = len(com)
        if P == 0 and K == 0:
            return None
        dev = prompt_tokens.device if P else com[0]["logits"].device
        uids = np.zeros(0, np.int64) if P == 0 else np.asarray(prompt_uids, dtype=np.int64)
        handles = np.zeros(0, np.int32)
        parts = []
        if P:
            last_logits = torch.empty((P, V), dtype=torch.float32, device=dev)
            handles = B.pc_prefill_shared(ctx, prompt_tokens, cu_lens, last_logits, stream)
            parts.append(last_logits)
        if K:
            parts.append(torch.stack([e["logits"] for e in com]))
        first_logits = parts[0] if len(parts) == 1 else torch.cat(parts)
        # ---- one decode batch: pilot sequences of this batch, then commit sequences of the selected prompts
        prow = np.repeat(np.arange(P, dtype=np.int32), npil)
        crow = np.repeat(np.arange(K, dtype=np.int32), ncom)
        seq_handles = np.concatenate([handles[prow], np.array([e["handle"] for e in com], np.int32)[crow]])
        logit_rows = np.concatenate([prow, P + crow]).astype(np.int32)
        c_uids = np.array([e["uid"] for e in com], np.int64)
        seq_uids = np.concatenate([_seq_uids(uids, range(npil)), _seq_uids(c_uids, range(npil, npil + ncom))])
        g = generate(ctx, seq_handles, logit_rows, first_logits, seq_uids, T, wl.temperature, self.seed, self.eos_id,
                     self.eos_bias, stream)
        n_p = P * npil
        out = dict(step=self.step_no, rows=n_p + K * ncom, decode_steps=g["steps_run"],
                   tokens_generated=int(g["lengths"].sum().item()))
        uid_d = torch.from_numpy(uids).to(dev)
        # ---- pilot outcome of this batch -> scheduler
        if P:
            prow_d = torch.from_numpy(prow).to(dev).long()
            pq_d = None if p_q is None else torch.from_numpy(np.asarray(p_q, np.float32)).to(dev)
            ru_d = None if reward_u is None else torch.from_numpy(np.asarray(reward_u, np.float32)).to(dev)
            pilot_r = synthetic_rewards(wl.reward, g["tokens"][:n_p], g["lengths"][:n_p], uid_d[prow_d],
                                        None if pq_d is None else pq_d[prow_d],
                                        None if ru_d is None else ru_d[:, :npil].reshape(-1))
            off = torch.arange(P + 1, dtype=torch.int32, device=dev) * npil
            p_hat = torch.empty(P, dtype=torch.float32, device=dev)
            B.pc_group_stats(pilot_r, off, None, None, p_hat, None, stream)
            p_hat_h = p_hat.cpu().numpy()                    # the step's read-back: P floats
            tags = np.arange(self.next_tag, self.next_tag + P, dtype=np.int64)
            self.next_tag += P
            cls, evict, counts = self.sched.pilot(uids, tags, p_hat_h)
            for q in range(P):
                if cls[q] == 1:
                    self.entries[int(tags[q])] = dict(
                        handle=int(handles[q]), uid=int(uids[q]), logits=last_logits[q],
                        pilot_r=pilot_r[q * npil:(q + 1) * npil], pilot_tokens=g["tokens"][q * npil:(q + 1) * npil],
                        reward_u=None if reward_u is None else np.asarray(reward_u[q], np.float32),
                        p_q=None if p_q is None else float(p_q[q]))
            dropped = handles[cls != 1]
            if len(dropped):
                B.pc_release(ctx, dropped, 1)
            out.update(pilot_tokens=g["tokens"][:n_p].view(P, npil, T), pilot_lens=g["lengths"][:n_p].view(P, npil),
                       pilot_rewards=pilot_r.view(P, npil), p_hat=p_hat_h, cls=cls, evict=evict, counts=counts)
        # ---- commit outcome of the prompts selected at the previous step -> advantages over pilot U commit
        if K:
            crow_d = torch.from_numpy(crow).to(dev).long()
            cu_d = torch.from_numpy(c_uids).to(dev)
            pq_c = ru_c = None
            if wl.reward == "bernoulli":
                pq_c = torch.tensor([e["p_q"] for e in com], dtype=torch.float32, device=dev)[crow_d]
                ru_c = torch.from_numpy(np.stack([e["reward_u"][npil:npil + ncom] for e in com])).to(dev).reshape(-1)
            commit_r = synthetic_rewards(wl.reward, g["tokens"][n_p:], g["lengths"][n_p:], cu_d[crow_d], pq_c, ru_c)
            union_r = torch.cat([torch.stack([e["pilot_r"] for e in com]), commit_r.view(K, ncom)], dim=1).contiguous()
            uoff = torch.arange(K + 1, dtype=torch.int32, device=dev) * (npil + ncom)
            adv = torch.zeros(K * (npil + ncom), dtype=torch.float32, device=dev)
            mu = torch.zeros(K, dtype=torch.float32, device=dev)
            sigma = torch.zeros(K, dtype=torch.float32, device=dev)
            B.pc_advantages(union_r.view(-1), uoff, self.eps, adv, mu, sigma, stream)
            out.update(commit_uids=c_uids, commit_tokens=g["tokens"][n_p:].view(K, ncom, T),
                       commit_lens=g["lengths"][n_p:].view(K, ncom), commit_rewards=commit_r.view(K, ncom),
                       commit_pilot_tokens=torch.stack([e["pilot_tokens"] for e in com]),
                       union_rewards=union_r, advantages=adv.view(K, npil + ncom), mu=mu, sigma=sigma)
            B.pc_release(ctx, np.array([e["handle"] for e in com], np.int32), 1)
            for t in self.pending:
                del self.entries[t]
        # ---- selection for the next step's commit pass; survivors that have waited too long are let go
        (s_uid, s_tag, s_age), (a_uid, a_tag) = self.sched.commit()
        for t in a_tag.tolist():
            e = self.entries.pop(int(t))
            B.pc_release(ctx, np.array([e["handle"]], np.int32), 1)
        self.pending = [int(t) for t in s_tag.tolist()]
        out.update(selected_uids=s_uid, selected_ages=s_age, aged_uids=a_uid)
        self.step_no += 1
        return out
