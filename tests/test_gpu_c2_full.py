"""GPU parity at the FULL size of the 1.5B-shaped workload, in the launch
configuration bench.py times (64 prompts x 256 tokens, 256 pilot sequences,
1024 new tokens, HIP-graph decode steps).  The oracle cannot redo 370k tokens
of a 1.5B model, so it checks sampled outputs one by one: one pilot sequence
is teacher-forced through the oracle's brute-force forward (all 1279 positions
of context, float64) and compared at sampled steps; everything that is cheap
(rewards, statistics, classes, commit set, advantages, counts) is compared
in full.
"""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import allocation, decoder, philox, sampler
from gpu_util import say, side_stream

pytestmark = pytest.mark.gpu


def test_c2_full_size_sampled_parity():
    import paper_2605_26606_amd as pc
    wl = workloads.WORKLOADS["C2"]
    m = wl.model
    P, Lp, T = wl.n_prompts, wl.prompt_len, wl.new_tokens
    say("C2 full size: building the model on the GPU")
    w = workloads.make_weights(m, wl.seed_weights, device="cuda")
    prompts = workloads.make_prompts(P, Lp, m.vocab, wl.seed_prompts)
    uids = workloads.make_prompt_uids(P)
    n_max = P * max(wl.n_pilot, wl.n_commit)
    kv_tokens = P * Lp + n_max * (T + 64) + 4096
    ctx = pc.Context(m, w, block_size=64, kv_pool_bytes=int(kv_tokens * m.kv_bytes_per_token() * 1.1),
                     max_slots=P + n_max + 8, max_ctx=Lp + T + 64, max_batch_rows=max(P * Lp, n_max))
    cu = (np.arange(P + 1) * Lp).astype(np.int32)
    toks = torch.from_numpy(prompts.reshape(-1).astype(np.int32)).cuda()
    seq = 4 * 17 + 2                                  # prompt 17, rollout 2
    with torch.cuda.stream(side_stream()):
        last = torch.empty((P, m.vocab), dtype=torch.float32, device="cuda")
        handles = pc.pc_prefill_shared(ctx, toks, cu, last)
        rows = np.repeat(np.arange(P, dtype=np.int32), wl.n_pilot)
        seq_uids = (rows.astype(np.int64) * 65536 + np.tile(np.arange(wl.n_pilot), P))
        say("pilot pass: 256 sequences x 1024 tokens")
        g = pc.generate(ctx, handles[rows], rows, last, seq_uids, T, wl.temperature, wl.seed_sampler,
                        keep_logits_rows=np.array([seq]))
        pc.pc_release(ctx, handles, 1)
    torch.cuda.synchronize()
    tokens = g["tokens"].cpu().numpy()
    assert tokens.shape == (P * wl.n_pilot, T) and tokens.min() >= 0 and tokens.max() < m.vocab
    gpu_logits = {t: g["logits"][t][0].cpu().numpy() for t in range(T)}

    # ---- allocation on the full batch, from the GPU's own rewards
    d = "cuda"
    r = (torch.from_numpy(tokens[:, -1].astype(np.int64)) % 7 == torch.from_numpy(rows.astype(np.int64)) % 7).float()
    off = torch.arange(P + 1, dtype=torch.int32) * wl.n_pilot
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
    wcls, wev, wci, _, wcnt = allocation.select_commit(want[2], wl.p_lower, wl.p_upper, wl.p_solve, 0)
    assert np.array_equal(cls.cpu().numpy(), wcls) and np.array_equal(ev.cpu().numpy(), wev)
    assert np.array_equal(cnt.cpu().numpy(), wcnt) and np.array_equal(ci.cpu().numpy()[:wcnt[0]], wci)
    say("classes: %d kept, %d easy, %d hard of %d prompts" % (wcnt[0], wcnt[2], wcnt[3], P))
    ctx.close()

    # ---- one sequence through the oracle, teacher-forced, float64
    steps = [0, 1, 2, 63, 255, 256, 257, 511, 767, 1022, 1023]
    q = rows[seq]
    full = np.concatenate([prompts[q], tokens[seq]])
    say("oracle: brute-force forward of %d positions (about a minute)" % (len(full) - 1))
    w_cpu = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in w.items()}
    want_logits = decoder.forward_full(m, w_cpu, full[:-1], rows=[Lp - 1 + t for t in steps])
    worst, sq, same, own = 0.0, 0.0, 0, 0
    for a, t in enumerate(steps):
        diff = want_logits[a] - gpu_logits[t]
        worst = max(worst, float(np.abs(diff).max()))
        sq += float((diff ** 2).mean())
        u = philox.sampling_uniform(wl.seed_sampler, int(seq_uids[seq]), t)
        same += int(sampler.sample_token(gpu_logits[t], wl.temperature, u)[0] == tokens[seq, t])
        own += int(sampler.sample_token(want_logits[a], wl.temperature, u)[0] == tokens[seq, t])
    rms = math.sqrt(sq / len(steps))
    say("max-abs logit error %.4g (rms %.3g) at %d sampled steps; tokens %d/%d from the GPU's logits, %d/%d from "
        "the oracle's own" % (worst, rms, len(steps), same, len(steps), own, len(steps)))
    assert np.abs(want_logits).max() > 0.1
    assert worst <= 2e-2
    assert same == len(steps)
