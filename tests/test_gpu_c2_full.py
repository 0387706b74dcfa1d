"""GPU parity at the FULL size of the 1.5B-shaped workload, in the launch
configuration bench.py times (64 prompts x 256 tokens, 256 pilot sequences,
commit pass on the kept prompts, 1024 new tokens, HIP-graph decode steps).

The oracle cannot redo 600k tokens of a 1.5B model, so it checks sampled
outputs one by one: three pilot sequences and one COMMIT-pass sequence are
teacher-forced through the oracle's brute-force forward (all 1279 positions
of context, float64) and compared at 52 steps each, spread over the context
(208 positions); everything that is cheap (rewards, statistics, classes,
commit set, advantages over the union groups, counts) is compared in full.

Token agreement: the oracle's sampler on the logits the GPU sampled from must
reproduce every token (that checks the sampler at this vocabulary).  Sampling
from the oracle's OWN logits agrees only as far as the logit error allows: for
the near-uniform next-token distribution of a random-init model a uniform
falls between the two sides' CDF boundaries with probability
~ 0.4 sqrt(V) rms(logit error), which at V = 151 936 and rms 2e-3 is about
0.3.  That expectation is asserted as a bound; the ">= 99 % of positions"
criterion itself is "parity unpinned" on this workload and is asserted where
it means something (peaked distributions, tests/test_gpu_decoder.py).
"""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import allocation, decoder, philox, sampler
from gpu_util import say, side_stream

pytestmark = pytest.mark.gpu


def _spread_steps(T, Lp, k):
    """k generation steps spread over the context, always with the first steps, the last ones and the
    steps around the first block boundary behind the prompt."""
    fixed = {0, 1, 2, 63, 64, 65, T - 2, T - 1}
    more = np.linspace(3, T - 3, k - len(fixed)).astype(int).tolist()
    steps = sorted(fixed | set(more))
    i = 5
    while len(steps) < k:          # linspace hit a fixed step: fill up
        if i not in steps:
            steps.append(i)
        i += 7
    return sorted(steps)[:k]


def _teacher_force(m, w_cpu, prompt, gen, gpu_logits, steps, uid, seed, temperature):
    """-> (max-abs error, sum of squared errors, count, tokens from the GPU's logits, tokens from the oracle's own)"""
    Lp = len(prompt)
    full = np.concatenate([prompt, gen])
    want = decoder.forward_full(m, w_cpu, full[:-1], rows=[Lp - 1 + t for t in steps])
    assert np.abs(want).max() > 0.1
    worst = sq = 0.0
    same = own = 0
    for a, t in enumerate(steps):
        diff = want[a] - gpu_logits[t]
        worst = max(worst, float(np.abs(diff).max()))
        sq += float((diff ** 2).sum())
        u = philox.sampling_uniform(seed, int(uid), t)
        same += int(sampler.sample_token(gpu_logits[t], temperature, u)[0] == gen[t])
        own += int(sampler.sample_token(want[a], temperature, u)[0] == gen[t])
    return worst, sq, want.size, same, own


def _collect(g, local_rows):
    """{local row: {step: logits}} from generate()'s kept logits"""
    out = {r: {} for r in local_rows}
    for t, lg, lr in zip(g["logits_steps"], g["logits"], g["logits_rows"]):
        lr = lr.cpu().numpy().tolist()
        lg = lg.cpu().numpy()
        for k, r in enumerate(lr):
            out[r][t] = lg[k]
    return out


def test_c2_full_size_sampled_parity():
    import paper_2605_26606_amd as pc
    wl = workloads.WORKLOADS["C2"]
    m = wl.model
    P, Lp, T, npil, ncom = wl.n_prompts, wl.prompt_len, wl.new_tokens, wl.n_pilot, wl.n_commit
    say("C2 full size: building the model on the GPU")
    w = workloads.make_weights(m, wl.seed_weights, device="cuda")
    prompts = workloads.make_prompts(P, Lp, m.vocab, wl.seed_prompts)
    uids = workloads.make_prompt_uids(P)
    n_max = P * max(npil, ncom)
    kv_tokens = P * Lp + n_max * (T + 64) + 4096
    ctx = pc.Context(m, w, block_size=64, kv_pool_bytes=int(kv_tokens * m.kv_bytes_per_token() * 1.1),
                     max_slots=P + n_max + 8, max_ctx=Lp + T + 64, max_batch_rows=max(P * Lp, n_max))
    cu = (np.arange(P + 1) * Lp).astype(np.int32)
    toks = torch.from_numpy(prompts.reshape(-1).astype(np.int32)).cuda()
    steps = _spread_steps(T, Lp, 52)
    pilot_seqs = [4 * 17 + 2, 4 * 0 + 0, 4 * 63 + 3]          # (prompt 17, rollout 2), (0, 0), (63, 3)
    d = "cuda"
    with torch.cuda.stream(side_stream()):
        last = torch.empty((P, m.vocab), dtype=torch.float32, device=d)
        handles = pc.pc_prefill_shared(ctx, toks, cu, last)
        rows = np.repeat(np.arange(P, dtype=np.int32), npil)
        seq_uids = (rows.astype(np.int64) * 65536 + np.tile(np.arange(npil), P))
        say("pilot pass: %d sequences x %d tokens" % (P * npil, T))
        g = pc.generate(ctx, handles[rows], rows, last, seq_uids, T, wl.temperature, wl.seed_sampler,
                        keep_logits_rows=np.array(pilot_seqs), keep_logits_steps=steps)
        torch.cuda.synchronize()
        tokens = g["tokens"].cpu().numpy()
        assert tokens.shape == (P * npil, T) and tokens.min() >= 0 and tokens.max() < m.vocab

        # ---- allocation on the full batch, from the GPU's own rewards
        r = (torch.from_numpy(tokens[:, -1].astype(np.int64)) % 7 == torch.from_numpy(rows.astype(np.int64)) % 7).float()
        off = torch.arange(P + 1, dtype=torch.int32) * npil
        n_pos = torch.empty(P, dtype=torch.int32, device=d)
        n_tot = torch.empty(P, dtype=torch.int32, device=d)
        p_hat = torch.empty(P, device=d)
        var = torch.empty(P, device=d)
        pc.pc_group_stats(r.to(d), off.to(d), n_pos, n_tot, p_hat, var)
        cls = torch.empty(P, dtype=torch.uint8, device=d)
        ev = torch.empty(P, dtype=torch.uint8, device=d)
        ci = torch.empty(P, dtype=torch.int32, device=d)
        si = torch.empty(P, dtype=torch.int32, device=d)
        cnt = torch.empty(4, dtype=torch.int32, device=d)
        pc.pc_select_commit(p_hat, P, wl.p_lower, wl.p_upper, wl.p_solve, 0, cls, ev, ci, si, cnt)
        torch.cuda.synchronize()
        want = allocation.group_stats(r.numpy(), off.numpy())
        assert np.array_equal(n_pos.cpu().numpy(), want[0]) and np.array_equal(p_hat.cpu().numpy(), want[2])
        assert np.array_equal(var.cpu().numpy(), want[3])
        wcls, wev, wci, _, wcnt = allocation.select_commit(want[2], wl.p_lower, wl.p_upper, wl.p_solve, 0)
        assert np.array_equal(cls.cpu().numpy(), wcls) and np.array_equal(ev.cpu().numpy(), wev)
        assert np.array_equal(cnt.cpu().numpy(), wcnt) and np.array_equal(ci.cpu().numpy()[:wcnt[0]], wci)
        K = int(wcnt[0])
        say("classes: %d kept, %d easy, %d hard of %d prompts" % (K, wcnt[2], wcnt[3], P))
        assert K >= 2

        # ---- commit pass on the kept prompts only (prefix KV reused), rollout indices n_pilot ..
        kept = wci
        crow = np.repeat(kept.astype(np.int32), ncom)
        c_uids = (crow.astype(np.int64) * 65536 + np.tile(np.arange(npil, npil + ncom), K))
        commit_seq = ncom * (K // 2) + 1                       # (kept prompt K/2, commit rollout 1)
        say("commit pass: %d sequences x %d tokens" % (K * ncom, T))
        gc = pc.generate(ctx, handles[crow], crow, last, c_uids, T, wl.temperature, wl.seed_sampler,
                         keep_logits_rows=np.array([commit_seq]), keep_logits_steps=steps)
        torch.cuda.synchronize()
        ctokens = gc["tokens"].cpu().numpy()
        pc.pc_release(ctx, handles, 1)
        assert pc.pc_kv_blocks(ctx)[0] == pc.pc_kv_blocks(ctx)[1]

        # ---- advantages over the union groups, at this size
        cr = (torch.from_numpy(ctokens[:, -1].astype(np.int64)) % 7 == torch.from_numpy(crow.astype(np.int64)) % 7).float()
        union = torch.cat([r.view(P, npil)[torch.from_numpy(kept).long()], cr.view(K, ncom)], dim=1).contiguous()
        uoff = torch.arange(K + 1, dtype=torch.int32) * (npil + ncom)
        adv = torch.empty(K * (npil + ncom), device=d)
        mu = torch.empty(K, device=d)
        sg = torch.empty(K, device=d)
        pc.pc_advantages(union.view(-1).to(d), uoff.to(d), 1e-6, adv, mu, sg)
        torch.cuda.synchronize()
        wadv, wmu, wsg = allocation.advantages(union.view(-1).numpy(), uoff.numpy())
        assert np.array_equal(adv.cpu().numpy(), wadv) and np.array_equal(mu.cpu().numpy(), wmu)
        assert np.array_equal(sg.cpu().numpy(), wsg)
        assert np.abs(adv.cpu().numpy().reshape(K, -1).sum(1)).max() < 1e-5
    sat = pc.pc_saturation_count(ctx)
    assert sat == 0, "%d activations left the half range" % sat
    ctx.close()

    # ---- four sequences through the oracle, teacher-forced, float64
    w_cpu = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in w.items()}
    del w
    pl = _collect(g, pilot_seqs)
    cl = _collect(gc, [commit_seq])
    cases = [("pilot", s, prompts[rows[s]], tokens[s], pl[s], seq_uids[s]) for s in pilot_seqs]
    cases.append(("commit", commit_seq, prompts[crow[commit_seq]], ctokens[commit_seq], cl[commit_seq], c_uids[commit_seq]))
    worst = sq = 0.0
    cnt_el = same = own = tot = 0
    for which, s, prompt, gen, gl, uid in cases:
        assert sorted(gl.keys()) == steps
        say("oracle: brute-force forward of %d positions for %s sequence %d (about a minute)" % (Lp + T - 1, which, s))
        wst, s2, c, sm, ow = _teacher_force(m, w_cpu, prompt, gen, gl, steps, uid, wl.seed_sampler, wl.temperature)
        say("  %s sequence %d: max-abs logit error %.4g; tokens %d/%d from the GPU's logits, %d/%d from the "
            "oracle's own" % (which, s, wst, sm, len(steps), ow, len(steps)))
        worst = max(worst, wst)
        sq += s2
        cnt_el += c
        same += sm
        own += ow
        tot += len(steps)
    rms = math.sqrt(sq / cnt_el)
    p_miss = 0.4 * math.sqrt(m.vocab) * rms
    say("C2 full size, %d positions: max-abs logit error %.4g (rms %.3g); tokens %d/%d from the GPU's logits, %d/%d "
        "from the oracle's own (expected miss rate %.2f)" % (tot, worst, rms, same, tot, own, tot, p_miss))
    assert tot >= 200
    assert worst <= 2e-2
    assert same == tot
    # agreement with the oracle's own logits: bounded by the logit error (see the module text), not 99 % here
    assert own >= tot * (1.0 - 1.5 * p_miss) - 3.0 * math.sqrt(tot * p_miss * (1.0 - min(p_miss, 0.5)))
    assert own >= 0.45 * tot           # measured floor: about two thirds agree at rms 2e-3


def test_c2_full_size_bf16_activations_against_their_own_bound():
    # PC_ACT_BF16 is outside the 2e-2 acceptance bound (every rounding point loses 2^-9 relative; 28 layers
    # drift by up to 1e-1); its stated bound is 1.5e-1 x max(1, max|logit|).  The sampler still has to
    # reproduce every token from the logits it was given.
    import paper_2605_26606_amd as pc
    wl = workloads.WORKLOADS["C2"]
    m = wl.model
    P, Lp, T, npil = wl.n_prompts, wl.prompt_len, wl.new_tokens, wl.n_pilot
    say("C2 full size, bf16 activations: pilot pass")
    w = workloads.make_weights(m, wl.seed_weights, device="cuda")
    prompts = workloads.make_prompts(P, Lp, m.vocab, wl.seed_prompts)
    n_max = P * npil
    kv_tokens = P * Lp + n_max * (T + 64) + 4096
    ctx = pc.Context(m, w, block_size=64, kv_pool_bytes=int(kv_tokens * m.kv_bytes_per_token() * 1.1),
                     max_slots=P + n_max + 8, max_ctx=Lp + T + 64, max_batch_rows=max(P * Lp, n_max), act_dtype="bf16")
    cu = (np.arange(P + 1) * Lp).astype(np.int32)
    toks = torch.from_numpy(prompts.reshape(-1).astype(np.int32)).cuda()
    steps = _spread_steps(T, Lp, 24)
    seq = 4 * 31 + 1
    with torch.cuda.stream(side_stream()):
        last = torch.empty((P, m.vocab), dtype=torch.float32, device="cuda")
        handles = pc.pc_prefill_shared(ctx, toks, cu, last)
        rows = np.repeat(np.arange(P, dtype=np.int32), npil)
        seq_uids = (rows.astype(np.int64) * 65536 + np.tile(np.arange(npil), P))
        g = pc.generate(ctx, handles[rows], rows, last, seq_uids, T, wl.temperature, wl.seed_sampler,
                        keep_logits_rows=np.array([seq]), keep_logits_steps=steps)
        pc.pc_release(ctx, handles, 1)
    torch.cuda.synchronize()
    assert pc.pc_saturation_count(ctx) == 0      # only the half path clamps
    tokens = g["tokens"].cpu().numpy()
    gl = _collect(g, [seq])[seq]
    ctx.close()
    w_cpu = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in w.items()}
    del w
    say("oracle: brute-force forward of %d positions (about a minute)" % (Lp + T - 1))
    worst, sq, c, same, own = _teacher_force(m, w_cpu, prompts[rows[seq]], tokens[seq], gl, steps, seq_uids[seq],
                                            wl.seed_sampler, wl.temperature)
    say("bf16 activations at C2 size: max-abs logit error %.4g (rms %.3g); tokens %d/%d from the GPU's logits, %d/%d "
        "from the oracle's own" % (worst, math.sqrt(sq / c), same, len(steps), own, len(steps)))
    assert worst <= 1.5e-1
    assert same == len(steps)
