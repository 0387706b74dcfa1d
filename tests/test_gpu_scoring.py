"""GPU parity of pc_score (teacher-forced log-probabilities of given
completions) against the scoring oracle, and consistency with the
log-probabilities the sampler hands on while generating."""
import numpy as np
import pytest
import torch

import workloads
from oracle import scoring
from gpu_util import make_ctx, say, side_stream

pytestmark = pytest.mark.gpu

C1 = workloads.WORKLOADS["C1"]
BF = workloads.scaled(C1, dtype="bf16", d_model=256, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ff=640,
                      vocab=2048, n_layers=3, rope_theta=1.0e6).model


def _score(model, w, seqs, plens, temperature, **kw):
    import paper_2605_26606_amd as pc
    ctx = make_ctx(model, w, **kw)
    cu = np.concatenate([[0], np.cumsum([len(s) for s in seqs])]).astype(np.int32)
    toks = torch.from_numpy(np.concatenate(seqs).astype(np.int32)).cuda()
    n_out = int(sum(len(s) - p for s, p in zip(seqs, plens)))
    out = torch.full((max(n_out, 1),), 7.0, dtype=torch.float32, device="cuda")
    with torch.cuda.stream(side_stream()):
        pc.pc_score(ctx, toks, cu, np.asarray(plens, np.int32), temperature, out)
        # a second call reuses the slots and blocks the first one gave back
        out2 = torch.empty_like(out)
        pc.pc_score(ctx, toks, cu, np.asarray(plens, np.int32), temperature, out2)
    torch.cuda.synchronize()
    assert pc.pc_kv_blocks(ctx)[0] == pc.pc_kv_blocks(ctx)[1]
    ctx.close()
    assert torch.equal(out, out2)
    return out.cpu().numpy()[:n_out]


@pytest.mark.parametrize("name,tol", [("fp32", 1e-4), ("f16", 2e-2)])
def test_scores_match_the_oracle(name, tol):
    model = C1.model if name == "fp32" else BF
    say("pc_score, %s model: ragged sequences, several chunks, temperature 1.0 and 0.7" % name)
    w = workloads.perturb_norm_gains(workloads.make_weights(model, 5), 2)
    rng = np.random.default_rng(3)
    lens = [40, 7, 33, 64, 2, 19, 50]
    plens = [12, 7, 1, 30, 1, 18, 25]              # one sequence has no completion at all
    seqs = [rng.integers(0, model.vocab, n) for n in lens]
    for T in (1.0, 0.7):
        got = _score(model, w, seqs, plens, T, block_size=32, kv_pool_bytes=64 << 20, max_slots=16, max_ctx=64,
                     max_batch_rows=96)           # 215 rows in chunks of at most 96
        want = np.concatenate([scoring.score(model, w, s, p, T) for s, p in zip(seqs, plens)])
        assert got.shape == want.shape
        err = np.abs(got - want).max()
        say("T=%.1f: %d completion tokens, max-abs log-probability error %.3g" % (T, len(want), err))
        assert err <= tol


def test_scores_equal_the_sampler_logprobs_of_generated_rollouts():
    # what the sampler reported while generating is what scoring the finished rollouts gives (same policy)
    import paper_2605_26606_amd as pc
    m = C1.model
    say("pc_score of generated rollouts vs the sampler's own log-probabilities (fp32)")
    w = workloads.make_weights(m, 1)
    ctx = make_ctx(m, w, block_size=32, kv_pool_bytes=64 << 20, max_slots=128, max_ctx=64, max_batch_rows=256)
    P, Lp, G, T = 6, 20, 3, 12
    prompts = workloads.make_prompts(P, Lp, m.vocab, 2)
    cu = (np.arange(P + 1) * Lp).astype(np.int32)
    toks = torch.from_numpy(prompts.reshape(-1).astype(np.int32)).cuda()
    with torch.cuda.stream(side_stream()):
        last = torch.empty((P, m.vocab), dtype=torch.float32, device="cuda")
        handles = pc.pc_prefill_shared(ctx, toks, cu, last)
        rows = np.repeat(np.arange(P, dtype=np.int32), G)
        uids = rows.astype(np.int64) * 65536 + np.tile(np.arange(G), P)
        g = pc.generate(ctx, handles[rows], rows, last, uids, T, 1.0, 3, keep_logprobs=True)
        pc.pc_release(ctx, handles, 1)
        full = np.concatenate([np.concatenate([prompts[rows[i]], g["tokens"][i].cpu().numpy()]) for i in range(P * G)])
        cu2 = (np.arange(P * G + 1) * (Lp + T)).astype(np.int32)
        out = torch.empty(P * G * T, dtype=torch.float32, device="cuda")
        pc.pc_score(ctx, torch.from_numpy(full.astype(np.int32)).cuda(), cu2, np.full(P * G, Lp, np.int32), 1.0, out)
    torch.cuda.synchronize()
    assert pc.pc_kv_blocks(ctx)[0] == pc.pc_kv_blocks(ctx)[1]
    ctx.close()
    got = out.cpu().numpy().reshape(P * G, T)
    want = g["logprobs"].cpu().numpy()
    assert np.abs(got - want).max() <= 2e-5


def test_argument_checks_leave_state_unchanged():
    import paper_2605_26606_amd as pc
    m = C1.model
    ctx = make_ctx(m, workloads.make_weights(m, 1), block_size=32, kv_pool_bytes=8 << 20, max_slots=4, max_ctx=64,
                   max_batch_rows=64)
    toks = torch.zeros(64, dtype=torch.int32, device="cuda")
    out = torch.zeros(64, dtype=torch.float32, device="cuda")
    free0 = pc.pc_kv_blocks(ctx)[0]
    for cu, pl in (([0, 10], [0]), ([0, 10], [11]), ([0, 0], [1]), ([0, 65], [3])):
        with pytest.raises((pc.PcError, ValueError)):
            pc.pc_score(ctx, torch.zeros(80, dtype=torch.int32, device="cuda"), cu, pl, 1.0, out)
    with pytest.raises(pc.PcError):
        pc.pc_score(ctx, toks, [0, 10], [3], 0.0, out)
    with pytest.raises(pc.PcError):                      # more sequences than slots
        pc.pc_score(ctx, toks, np.arange(6) * 8, [1] * 5, 1.0, out)
    assert pc.pc_kv_blocks(ctx)[0] == free0
    pc.pc_score(ctx, toks, [0, 10, 30], [3, 5], 1.0, out)
    torch.cuda.synchronize()
    assert pc.pc_kv_blocks(ctx)[0] == free0
    ctx.close()
