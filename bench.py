#!/usr/bin/env python3
"""Benchmark: generated rollout tokens/s of one full Pilot-Commit sampling
step (shared-prefix prefill, pilot rollouts, group statistics, selection,
commit rollouts on the kept prompts, advantages) at the 1.5B shape on ONE
MI355X, with the decode-attention kernel priced against the HBM roofline and
the CPU oracle timed beside it on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints one JSON line.  A "step" is one pass of the whole path over one batch
of synthetic prompts (64 prompts x 256 tokens, pilot 4 + commit 4 rollouts,
1024 new tokens each).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

# HBM traffic of one launch of the timed kernel, from the profiler's FETCH_SIZE / WRITE_SIZE counters
# (profiles/attention_decode_c2_hbm_counters.txt).  Taken with the standalone kernel driver: same kernel,
# grid and shapes (256 sequences in groups of 4, 256 prefix + 512 generated tokens = the mean context of
# the launches timed here).  Each counter is scaled by what it reads for a plain 1 GiB copy.  The figure
# is only reported while the kernel source is the one the counters were taken on.
ATTN_COUNTERS = {"source": "paper_2605_26606_amd/csrc/attention.hip",
                 "sha256": "35566b3ef867b4154273fdf13e4146a366baf02035906a15f2082e3df47a61ee",
                 "seqs": 256, "prompt_len": 256, "mean_generated": 512,
                 "fetch_kib": 74216.6, "fetch_scale": 1048576.0 / 524300.9,
                 "write_kib": 768.0, "write_scale": 1048576.0 / 1048576.0}


def counter_traffic_bytes(n_seqs, prompt_len, mean_generated):
    import hashlib
    c = ATTN_COUNTERS
    try:
        with open(os.path.join(ROOT, c["source"]), "rb") as f:
            same = hashlib.sha256(f.read()).hexdigest() == c["sha256"]
    except OSError:
        same = False
    if not same or (n_seqs, prompt_len) != (c["seqs"], c["prompt_len"]) or abs(mean_generated - c["mean_generated"]) > 1:
        return None
    return int((c["fetch_kib"] * c["fetch_scale"] + c["write_kib"] * c["write_scale"]) * 1024)


def decode_bytes_per_step(model, n_prompts_active, prompt_len, n_seqs, t):
    """Algorithmic HBM bytes of decode step t (the step that feeds generated token t-1):
    all weights once + prefix KV once per prompt + generated KV per sequence (the appended
    token included).  Logit traffic is excluded."""
    w = (model.body_params() + model.lm_head_params()) * model.elem_bytes()
    kv = (n_prompts_active * prompt_len + n_seqs * t) * model.kv_bytes_per_token()
    return w + kv


def attention_bytes_per_launch(model, n_prompts_active, prompt_len, n_seqs, t):
    """Algorithmic bytes of ONE decode-attention launch (one layer) at step t."""
    per_tok = 2 * model.n_kv_heads * model.head_dim * model.elem_bytes()
    return (n_prompts_active * prompt_len + n_seqs * t) * per_tok


def cpu_baseline(wl, w_dev, prompts, uids, seed):
    """Times the oracle, as it stands, on bounded samples of the same workload: prefill and decode separately, with
    all host threads and with one."""
    import numpy as np
    import torch
    from oracle import philox, sampler
    from oracle.decoder import CachedDecoder
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [torch.get_num_threads()])
    except Exception:
        threadpool_limits = None
        threads = torch.get_num_threads()
    w_cpu = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in w_dev.items()}

    def run(n_prefill, n_roll, n_new):
        t0 = time.perf_counter()
        base = CachedDecoder(wl.model, w_cpu)
        first = base.extend(prompts[0][:n_prefill])
        t1 = time.perf_counter()
        for j in range(n_roll):
            dec, logits = base.clone(), first
            uid = philox.seq_uid(int(uids[0]), j)
            for t in range(n_new):
                tok, _ = sampler.sample_token(logits, wl.temperature, philox.sampling_uniform(seed, uid, t))
                logits = dec.extend([tok])          # n_new decode forwards per rollout
        t2 = time.perf_counter()
        return n_prefill / (t1 - t0), n_roll * n_new / (t2 - t1), n_roll * n_new / (t2 - t0), t2 - t0

    n_roll, n_new = 2, 4
    pre, dec, both, secs = run(wl.prompt_len, n_roll, n_new)
    out = {"value": both, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": "1 prompt x %d tokens prefilled once, %d rollouts x %d decode forwards, float64 numpy (%.1f s); value "
                     "= generated tokens / (prefill + decode) time" % (wl.prompt_len, n_roll, n_new, secs),
           "prefill_tokens_per_s": round(pre, 2), "decode_tokens_per_s": round(dec, 3)}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            torch_threads = torch.get_num_threads()
            torch.set_num_threads(1)
            pre1, dec1, _, secs1 = run(32, 1, 2)
            torch.set_num_threads(torch_threads)
        out["one_thread"] = {"prefill_tokens_per_s": round(pre1, 2), "decode_tokens_per_s": round(dec1, 3),
                             "sample": "32 prompt tokens, 1 rollout x 2 decode forwards at a context of 32 (%.1f s)" % secs1}
    return out


def parity_sample(pc, ctx, wl, w_dev, toks, cu, prompts, uids, seed, stream, span=0, say=None):
    """One pilot sequence of a fresh pilot pass, teacher-forced through the oracle at 12 steps spread over the context
    (over its first `span` generated tokens when span > 0: the oracle's cost grows with the context, and for the
    8B shape the whole one takes it a quarter of an hour): max-abs logit error and the two token agreements (the
    oracle's sampler on the GPU's logits / on its own)."""
    import numpy as np
    import torch
    from oracle import decoder, philox, sampler
    m, P, Lp, T = wl.model, wl.n_prompts, wl.prompt_len, wl.new_tokens
    Ts = min(T, span) if span > 0 else T
    steps = sorted(set([0, 1, Ts - 1] + np.linspace(2, Ts - 2, 9).astype(int).tolist()))
    seq = wl.n_pilot * (P // 2) + 1
    with torch.cuda.stream(stream):
        last = torch.empty((P, m.vocab), dtype=torch.float32, device=toks.device)
        handles = pc.pc_prefill_shared(ctx, toks, cu, last, stream)
        rows = np.repeat(np.arange(P, dtype=np.int32), wl.n_pilot)
        seq_uids = (np.asarray(uids, np.int64)[:, None] * 65536 + np.arange(wl.n_pilot)[None, :]).reshape(-1)
        g = pc.generate(ctx, handles[rows], rows, last, seq_uids, Ts, wl.temperature, seed, -1, 0.0, stream,
                        keep_logits_rows=np.array([seq]), keep_logits_steps=steps)
        pc.pc_release(ctx, handles, 1)
    torch.cuda.synchronize()
    gen = g["tokens"][seq].cpu().numpy()
    gl = {t: lg[0].cpu().numpy() for t, lg in zip(g["logits_steps"], g["logits"])}
    w_cpu = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in w_dev.items()}
    full = np.concatenate([prompts[rows[seq]], gen[:Ts]])
    want = decoder.forward_full(m, w_cpu, full[:-1], rows=[Lp - 1 + t for t in steps],
                                on_layer=(lambda l: say("oracle: layer %d of %d" % (l + 1, m.n_layers))) if say else None)
    worst = sq = 0.0
    same = own = 0
    for a, t in enumerate(steps):
        diff = want[a] - gl[t]
        worst = max(worst, float(np.abs(diff).max()))
        sq += float((diff ** 2).mean())
        u = philox.sampling_uniform(seed, int(seq_uids[seq]), t)
        same += int(sampler.sample_token(gl[t], wl.temperature, u)[0] == gen[t])
        own += int(sampler.sample_token(want[a], wl.temperature, u)[0] == gen[t])
    return {"positions": len(steps), "context": "%d prompt + first %d generated tokens" % (Lp, Ts),
            "max_abs_logit_error": round(worst, 5),
            "rms_logit_error": round(float(np.sqrt(sq / len(steps))), 6),
            "tokens_from_gpu_logits": same, "tokens_from_oracle_logits": own,
            "note": "one pilot sequence of the timed workload, teacher-forced through the float64 oracle; agreement from "
                    "the oracle's own logits is bounded by ~1 - 0.4 sqrt(V) rms for the near-uniform distributions of a "
                    "random-init model"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--new-tokens", type=int, default=0, help="override the workload's new tokens (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle check of one sequence of the workload")
    ap.add_argument("--parity-span", type=int, default=0,
                    help="check only the first N generated tokens of that sequence (large models: the oracle is slow)")
    ap.add_argument("--verbose", action="store_true", help="(kept for old command lines: phases are always reported on stderr)")
    ap.add_argument("--eos-bias", default="0",
                    help="logit bias on the EOS id of the workloads that stop on EOS: a number, or 'ragged' for "
                         "ln(V / (T/2)), i.e. a stop hazard of about 2/T per step (mean length near T/2); "
                         "0 is the literal reading (one id in V almost never fires)")
    ap.add_argument("--b-t", type=int, default=0,
                    help="cap on the prompts committed per step (Section 3.3 b_t); also bounds the KV pool, which "
                         "otherwise is sized for every prompt being kept")
    ap.add_argument("--time-every", type=int, default=64)
    ap.add_argument("--act", default="f16", choices=["f16", "bf16"],
                    help="activation / KV type of 16-bit models: IEEE half (the accepted configuration) or bfloat16 "
                         "(outside the 2e-2 logit bound at 28 layers; measured for comparison)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch decode steps eagerly (for counter runs: the profiler's counter mode and HIP graphs "
                         "do not go together)")
    ap.add_argument("--binding-steps", type=int, default=4,
                    help="after the timed steps, also run this many sampling batches through the bound pipeline "
                         "(commit pass of step t-1 in one decode batch with the pilot pass of step t); 0 = skip")
    ap.add_argument("--no-gemm-timing", action="store_true", help="skip the per-launch timing of the decode GEMMs")
    ap.add_argument("--no-score", action="store_true",
                    help="skip the scoring leg (pc_score over the last step's pilot rollouts)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (the known-size reference of the counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this library runs on one GPU; --gpus %d is not supported (no multi-GPU path "
                         "exists in this library)\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    import paper_2605_26606_amd as pc

    wl = workloads.WORKLOADS[args.workload]
    if args.new_tokens:
        wl = workloads.scaled(wl, new_tokens=args.new_tokens)
    if args.b_t:
        wl = workloads.scaled(wl, b_t=args.b_t)
    m = wl.model
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = workloads.make_weights(m, wl.seed_weights, device=dev)
    prompts = workloads.make_prompts(wl.n_prompts, wl.prompt_len, m.vocab, wl.seed_prompts)
    uids = workloads.make_prompt_uids(wl.n_prompts)
    P, Lp, T = wl.n_prompts, wl.prompt_len, wl.new_tokens
    bound = args.binding_steps > 0
    # unbound: one pass at a time; bound: pilot and commit sequences decode together, two batches of prompts alive
    P_commit = min(P, wl.b_t) if wl.b_t > 0 else P
    n_max = P * wl.n_pilot + P_commit * wl.n_commit if bound else max(P * wl.n_pilot, P_commit * wl.n_commit)
    n_prompts_alive = 2 * P if bound else P
    kv_tokens = n_prompts_alive * Lp + n_max * (T + 64) + 4096
    if not args.no_score:   # the scoring leg runs every pilot rollout (prompt + completion) through the forward
        kv_tokens = max(kv_tokens, P * wl.n_pilot * (Lp + T + 64) + 4096)
    # The pool is sized for every prompt being kept, but never beyond what the GPU has left next to the caller's
    # weights, the library's own copies, the activation buffers and the logits; a pass whose sequences do not fit is
    # cut into waves (rollout.generate).
    want_pool = int(kv_tokens * m.kv_bytes_per_token() * 1.1)
    free_b, _total_b = torch.cuda.mem_get_info()
    rows_max = max(P * Lp, n_max)
    qd_, kvd_ = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    lib_bytes = (m.body_params() + m.lm_head_params()) * 2
    act_bytes = rows_max * (4 * m.d_model + 4 * (qd_ + 2 * kvd_) + 2 * max(m.d_model, qd_) + 4 * qd_ + 2 * m.d_ff) + (64 << 20)
    logit_bytes = 3 * n_max * m.vocab * 4 + (1024 * m.vocab * 4 if not args.no_score else 0)
    pool = min(want_pool, int(free_b - lib_bytes - act_bytes - logit_bytes - (8 << 30)))
    if pool < want_pool:
        say_early = "KV pool %.1f GB of the %.1f GB an all-kept step would take: passes may run in waves" % (
            pool / 2 ** 30, want_pool / 2 ** 30)
        sys.stderr.write("[bench] " + say_early + "\n")
    ctx = pc.Context(m, w, block_size=64, kv_pool_bytes=pool,
                     max_slots=n_prompts_alive + n_max + 8, max_ctx=Lp + T + 64, max_batch_rows=rows_max,
                     act_dtype=args.act)
    if args.no_graph:
        pc.pc_set_option(ctx, pc.PC_OPT_USE_GRAPH, 0)
    cu = (np.arange(P + 1) * Lp).astype(np.int32)
    toks = torch.from_numpy(prompts.reshape(-1).astype(np.int32)).to(dev)
    eos_id = workloads.make_eos_id(m.vocab, wl.seed_eos) if wl.eos else -1
    import math
    eos_bias = (math.log(m.vocab / (wl.new_tokens / 2.0)) if args.eos_bias == "ragged" else float(args.eos_bias)) \
        if wl.eos else 0.0
    p_q = workloads.make_success_probs(P, wl.seed_reward) if wl.reward == "bernoulli" else None
    ru = workloads.make_reward_uniforms(P, wl.n_pilot + wl.n_commit, wl.seed_reward) \
        if wl.reward == "bernoulli" else None
    stream = torch.cuda.Stream()

    def say(msg):   # a line per completed phase on stderr (a long workload is silent for minutes otherwise)
        sys.stderr.write("[bench %.0f s] %s\n" % (time.perf_counter() - t_start, msg))
        sys.stderr.flush()

    t_start = time.perf_counter()

    def one_step(seed, timed_steps=None, timings=None):
        with torch.cuda.stream(stream):
            return pc.pilot_commit_step(ctx, wl, toks, cu, uids, seed, eos_id, eos_bias, p_q, ru,
                                        time_class=pc.PC_KERNEL_ATTN_DECODE if timed_steps is not None else -1,
                                        time_every=args.time_every if timed_steps is not None else 0,
                                        timed_steps=timed_steps, timings=timings, log=say)

    for i in range(args.warmup):
        one_step(wl.seed_sampler + 1000 + i)
    torch.cuda.synchronize()
    pc.pc_timing_read(ctx, reset=True)

    timed_steps, timings, outs = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        tm = {}
        outs.append(one_step(wl.seed_sampler + i, timed_steps, tm))
        timings.append(tm)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    tokens = sum(o["tokens_generated"] for o in outs)
    attn_ms, attn_launches, empty_ms, empty_pairs = pc.pc_timing_read(ctx, reset=True)
    # algorithmic bytes of the timed attention launches (every layer of every timed step)
    attn_bytes = sum(attention_bytes_per_launch(m, pa, Lp, n, t) for (_, t, n, pa) in timed_steps) * m.n_layers
    roof = None
    if attn_launches > 0 and attn_ms > 0:
        bracket_ms = empty_ms / empty_pairs if empty_pairs else 0.0   # what an event pair around nothing reads
        avg_ms = max(attn_ms / attn_launches - bracket_ms, 1e-6)
        achieved = attn_bytes / attn_launches / (avg_ms * 1e-3) / 1e9
        pilot_t = [t for (which, t, _, _) in timed_steps if which == "pilot"]
        traffic = counter_traffic_bytes(P * wl.n_pilot, Lp, sum(pilot_t) / max(1, len(pilot_t))) \
            if len(pilot_t) == len(timed_steps) and args.act == "f16" else None
        roof = {"kernel": "attention_decode_mfma_kernel<%s, direct, 4 waves> (pilot pass, %d sequences)" % (args.act, P * wl.n_pilot), "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "avg_launch_us": round(avg_ms * 1e3, 2), "event_bracket_us": round(bracket_ms * 1e3, 2),
                "launches_timed": int(attn_launches),
                "bytes_per_launch": int(attn_bytes / attn_launches)}
    # whole decode loop against the HBM roofline (weights + KV per step, prefix counted once per prompt)
    dec_bytes = dec_ms = 0.0
    for o, tm in zip(outs, timings):
        K = int(o["counts"][0])
        for t in range(1, T):
            dec_bytes += decode_bytes_per_step(m, P, Lp, P * wl.n_pilot, t)
            if K:
                dec_bytes += decode_bytes_per_step(m, K, Lp, K * wl.n_commit, t)
        dec_ms += tm.get("pilot_ms", 0.0) + tm.get("commit_ms", 0.0)
    ragged = eos_id >= 0 and eos_bias != 0.0
    if ragged:   # sequences leave the batch early: the full-length byte counts above do not describe this run
        roof, dec_bytes = None, 0.0
    prefill_flops = 2.0 * m.body_params() * P * Lp + 2.0 * m.lm_head_params() * P \
        + 2.0 * m.n_layers * P * m.n_q_heads * m.head_dim * Lp * Lp
    prefill_ms = sum(tm.get("prefill_ms", 0.0) for tm in timings) / max(1, len(timings))
    result = {
        "metric": "rollout tokens/s on 1 MI355X (1.5B shape, G=8); decode HBM GB/s % of peak",
        "value": round(tokens / dt, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(dt * 1e3 / max(1, args.steps), 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        # matrix-core inputs: IEEE half copies of the bf16 weights and half activations / KV, fp32 accumulation
        "dtype": args.act if m.dtype == "bf16" else m.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d prompts x %d tokens, pilot %d + commit %d rollouts on kept prompts, %d new "
                               "tokens, L%d d%d %dq/%dkv hd%d ff%d V%d, random init" %
                               (wl.name, P, Lp, wl.n_pilot, wl.n_commit, T, m.n_layers, m.d_model, m.n_q_heads,
                                m.n_kv_heads, m.head_dim, m.d_ff, m.vocab),
                   "eos_logit_bias": round(eos_bias, 3),
                   "kv_pool_GB": round(pool / 2 ** 30, 1),
                   "kept_prompts": [int(o["counts"][0]) for o in outs],
                   "rollouts": [int(o["rollouts"]) for o in outs]},
        # the whole decode loop first, then its dominant kernel
        "decode": {"ms": round(dec_ms, 1), "steps": sum(o["decode_steps"] for o in outs),
                   "algorithmic_GBps": None if ragged else round(dec_bytes / max(dec_ms, 1e-9) / 1e6, 1),
                   "frac_hbm": None if ragged else round(dec_bytes / max(dec_ms, 1e-9) / 1e6 / HBM_PEAK_GBPS, 4)},
        "roofline": roof,
        "prefill": {"ms": round(prefill_ms, 2), "TFLOPs": round(prefill_flops / max(prefill_ms, 1e-9) / 1e9, 1),
                    "frac_mfma": round(prefill_flops / max(prefill_ms, 1e-9) / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)},
    }
    if bound:
        # the same work re-scheduled (Section 3.4 binding): fresh prompts every step, commit pass of the previous
        # step's kept prompts in the same decode batch as this step's pilot pass; one extra pass drains the last commit
        batches = []
        for b in range(args.binding_steps):
            pr = workloads.make_prompts(P, Lp, m.vocab, wl.seed_prompts + 100 + b)
            batches.append((torch.from_numpy(pr.reshape(-1).astype(np.int32)).to(dev),
                            workloads.make_prompt_uids(P, first=10000 * (b + 1))))
        with torch.cuda.stream(stream):
            pipe = pc.BoundPipeline(ctx, wl, wl.seed_sampler + 7, eos_id, eos_bias)
            torch.cuda.synchronize()
            marks, info = [time.perf_counter()], []
            for tk, uid_b in batches + [(None, None)]:
                o = pipe.step(tk, None if tk is None else cu, uid_b,
                              p_q=p_q, reward_u=ru) if tk is not None else pipe.step(None, None, None)
                torch.cuda.synchronize()
                marks.append(time.perf_counter())
                if o is not None:
                    info.append((o["rows"], o["tokens_generated"], marks[-1] - marks[-2]))
                    say("bound pipeline: pass %d done (%d rows)" % (len(info), o["rows"]))
            pipe.close()
        tot_tok = sum(i[1] for i in info)
        mid = info[1:-1] if len(info) > 2 else info
        result["binding"] = {
            "value": round(tot_tok / (marks[-1] - marks[0]), 1), "unit": "tokens/s",
            "sampling_batches": args.binding_steps, "passes": len(info),
            "steady_tokens_per_s": round(sum(i[1] for i in mid) / sum(i[2] for i in mid), 1),
            "rows_per_pass": [i[0] for i in info], "ms_per_pass": [round(i[2] * 1e3, 1) for i in info],
            "note": "ramp-up (pilot only) and drain (commit only) passes included in value, excluded from steady"}
    if not args.no_score and outs:
        # teacher-forced scoring of the pilot rollouts just generated (the per-token factors of Eq. 2's ratio):
        # one forward over prompt + completion of every rollout, log-softmax at the next token
        o = outs[-1]
        npil = wl.n_pilot
        comp = o["pilot_tokens"].reshape(P * npil, T)
        lens = o["pilot_lens"].reshape(-1).cpu().numpy()
        pr_d = toks.view(P, Lp).repeat_interleave(npil, dim=0)
        seqs = torch.cat([pr_d, comp], dim=1)
        keep = torch.arange(Lp + T, device=dev)[None, :] < (Lp + torch.from_numpy(lens).to(dev))[:, None]
        packed = seqs[keep].contiguous()
        cu_s = np.concatenate([[0], np.cumsum(Lp + lens)]).astype(np.int32)
        n_sc = int(lens.sum())
        lp_out = torch.empty(n_sc, dtype=torch.float32, device=dev)
        with torch.cuda.stream(stream):
            pc.pc_score(ctx, packed, cu_s, np.full(P * npil, Lp, np.int32), wl.temperature, lp_out)   # allocates once
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            pc.pc_score(ctx, packed, cu_s, np.full(P * npil, Lp, np.int32), wl.temperature, lp_out)
            torch.cuda.synchronize()
            dt_s = time.perf_counter() - t1
        rows_s = int(cu_s[-1])
        flops = 2.0 * m.body_params() * rows_s + 2.0 * m.lm_head_params() * n_sc \
            + sum(2.0 * m.n_layers * m.n_q_heads * m.head_dim * float(l) * float(l) for l in (Lp + lens))
        result["scoring"] = {"value": round(n_sc / dt_s, 1), "unit": "scored tokens/s", "sequences": P * npil,
                             "rows": rows_s, "ms": round(dt_s * 1e3, 1), "TFLOPs": round(flops / dt_s / 1e12, 1),
                             "frac_mfma": round(flops / dt_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                             "mean_logprob": round(float(lp_out.mean().item()), 4)}
        say("scoring pass done")
    if not args.no_gemm_timing:
        # per-launch time of the decode step's projection GEMMs at the pilot batch size (outside the timed region):
        # a few eagerly launched decode steps with an event pair around every launch of one class, as for the
        # attention figure above; priced against both rooflines (weights + activations in + result out, once each)
        n = P * wl.n_pilot
        qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
        shapes = {"qkv": (pc.PC_KERNEL_GEMM_QKV, qd + 2 * kvd, m.d_model, 4), "wo": (pc.PC_KERNEL_GEMM_WO, m.d_model, qd, 4),
                  "gate_up_swiglu": (pc.PC_KERNEL_GEMM_GATE_UP, 2 * m.d_ff, m.d_model, 1),
                  "down": (pc.PC_KERNEL_GEMM_DOWN, m.d_model, m.d_ff, 4), "lm_head": (pc.PC_KERNEL_GEMM_LM_HEAD, m.vocab, m.d_model, 4)}
        gem = {"rows": n}
        with torch.cuda.stream(stream):
            last = torch.empty((P, m.vocab), dtype=torch.float32, device=dev)
            handles = pc.pc_prefill_shared(ctx, toks, cu, last, stream)
            rows = np.repeat(np.arange(P, dtype=np.int32), wl.n_pilot)
            seq_uids = (np.asarray(uids, np.int64)[:, None] * 65536 + np.arange(wl.n_pilot)[None, :]).reshape(-1)
            for name, (cls, N, K, out_bytes) in shapes.items():
                torch.cuda.synchronize()
                pc.pc_timing_read(ctx, reset=True)
                pc.generate(ctx, handles[rows], rows, last, seq_uids, 14, wl.temperature, wl.seed_sampler + 99, -1, 0.0,
                            stream, time_class=cls, time_every=2)
                torch.cuda.synchronize()
                ms, cnt, ems, ecnt = pc.pc_timing_read(ctx, reset=True)
                if cnt == 0:
                    continue
                us = max(ms / cnt - (ems / ecnt if ecnt else 0.0), 1e-6) * 1e3
                byts = 2.0 * N * K + 2.0 * n * K + float(out_bytes) * n * N
                flops = 2.0 * n * N * K
                say("decode GEMM timing: %s done" % name)
                gem[name] = {"us": round(us, 2), "launches_timed": int(cnt), "GBps": round(byts / us / 1e3, 1),
                             "frac_hbm": round(byts / us / 1e3 / HBM_PEAK_GBPS, 4), "TFLOPs": round(flops / us / 1e6, 1),
                             "frac_mfma": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
            pc.pc_release(ctx, handles, 1)
        result["decode_gemms"] = gem
    if args.calibrate_copy:   # rocprofv3 --pmc runs scale FETCH_SIZE / WRITE_SIZE by what this copy reads
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_parity and m.dtype == "bf16":   # (its own pilot pass, generated without an EOS id)
        result["parity"] = parity_sample(pc, ctx, wl, w, toks, cu, prompts, uids, wl.seed_sampler + 5, stream,
                                         span=args.parity_span,
                                         say=say if m.n_layers * m.d_model * (Lp + T) > 28 * 1536 * 1500 else None)
        say("parity sample done")
    result["saturated_stores"] = pc.pc_saturation_count(ctx)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, w, prompts, uids, wl.seed_sampler)
    ctx.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
