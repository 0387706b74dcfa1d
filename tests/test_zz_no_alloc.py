"""pc_decode_step_static (the decode step that allocates nothing: eager
launches, scratch in the library's static device array) against
pc_decode_step on identical cache contents, called through the C ABI: two
calls in a row, the second on a smaller batch; same kernels and launch shapes,
so the logits must be bit-equal (and with them inside the logit tolerance of
the parity tests: 1e-4 fp32, 2e-2 for 16-bit models).  Oversized batches are
refused with a clear error before anything is launched."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import make_ctx, say, side_stream

pytestmark = pytest.mark.gpu

C1 = workloads.WORKLOADS["C1"]
BF = workloads.scaled(C1, dtype="bf16", d_model=256, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ff=640,
                      vocab=2048, n_layers=3, rope_theta=1.0e6).model
# wide enough that the down projection is cut into K slices while decoding (the slices are scratch)
BF8 = workloads.scaled(C1, dtype="bf16", d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ff=8192,
                       vocab=4096, n_layers=2, rope_theta=1.0e6).model


@pytest.mark.parametrize("name,model,lens,tol", [("fp32", C1.model, [20, 33, 7], 1e-4),
                                                 ("f16", BF, [70, 33, 128], 2e-2),
                                                 ("f16-split-k", BF8, [100, 31, 600], 2e-2)])
def test_static_decode_step_equals_decode_step(name, model, lens, tol):
    import paper_2605_26606_amd as pc
    say("pc_decode_step_static vs pc_decode_step, %s model" % name)
    w = workloads.perturb_norm_gains(workloads.make_weights(model, 3), 10)
    toks, cu = workloads.make_ragged_prompts(lens, model.vocab, 8)
    ctx = make_ctx(model, w, block_size=32, kv_pool_bytes=256 << 20, max_slots=64, max_ctx=1024, max_batch_rows=1024)
    G, V = 4, model.vocab
    rng = np.random.default_rng(1)
    with torch.cuda.stream(side_stream()):
        last = torch.empty((len(lens), V), dtype=torch.float32, device="cuda")
        handles = pc.pc_prefill_shared(ctx, torch.from_numpy(toks).cuda(), cu, last)
        rows = np.repeat(np.arange(len(lens), dtype=np.int32), G)
        a = pc.pc_fork(ctx, handles[rows], 8)          # the same prompts forked twice: two identical sets of sequences
        b = pc.pc_fork(ctx, handles[rows], 8)
        n = len(rows)
        la = torch.full((n, V), 7.0, dtype=torch.float32, device="cuda")
        lb = torch.full((n, V), -7.0, dtype=torch.float32, device="cuda")
        for call, m in enumerate((n, 5, 5)):            # the second and third call on a smaller batch
            tk = torch.from_numpy(rng.integers(0, V, m).astype(np.int32)).cuda()
            pc.pc_decode_step(ctx, a[:m], tk, la)
            pc.pc_decode_step_static(ctx, b[:m], tk, lb)
            torch.cuda.synchronize()
            ga, gb = la[:m].cpu().numpy(), lb[:m].cpu().numpy()
            assert np.isfinite(ga).all() and np.abs(ga).max() > 0.01
            worst = float(np.abs(ga - gb).max())
            say("  call %d (%d sequences): max-abs difference %.3g" % (call, m, worst))
            assert worst <= tol
            assert np.array_equal(ga, gb)
        pc.pc_release(ctx, a, 0)
        pc.pc_release(ctx, b, 0)
        pc.pc_release(ctx, handles, 1)
    torch.cuda.synchronize()
    assert pc.pc_kv_blocks(ctx)[0] == pc.pc_kv_blocks(ctx)[1]
    ctx.close()


def test_static_decode_step_refuses_what_does_not_fit():
    import paper_2605_26606_amd as pc
    w = workloads.make_weights(BF, 3)
    # 600 sequences x 2048 q/k/v columns x 8 slices x 4 bytes = 39 MB > the 32 MiB array
    ctx = make_ctx(BF, w, block_size=64, kv_pool_bytes=256 << 20, max_slots=700, max_ctx=128, max_batch_rows=640)
    toks = torch.zeros(64, dtype=torch.int32, device="cuda")
    last = torch.empty((1, BF.vocab), device="cuda")
    h = pc.pc_prefill_shared(ctx, toks, [0, 64], last)
    s = pc.pc_fork(ctx, [h[0]] * 600, 1)
    tk = torch.zeros(600, dtype=torch.int32, device="cuda")
    lg = torch.zeros((600, BF.vocab), device="cuda")
    with pytest.raises(pc.PcError) as e:
        pc.pc_decode_step_static(ctx, s, tk, lg)
    assert e.value.code == -1 and "static array" in str(e.value)
    torch.cuda.synchronize()
    assert not lg.any()                                # nothing was launched
    pc.pc_decode_step_static(ctx, s[:300], tk, lg)     # what fits still runs, and the refused call changed nothing
    pc.pc_decode_step(ctx, s[300:], tk, lg[300:])
    torch.cuda.synchronize()
    assert torch.isfinite(lg).all() and lg[:300].abs().max() > 0
    # identical sequences (same prompt, same token) give identical logits, whichever entry point ran them
    assert torch.equal(lg[0], lg[299]) and torch.allclose(lg[0], lg[599], atol=2e-2)
    pc.pc_release(ctx, s, 0)
    pc.pc_release(ctx, h, 1)
    ctx.close()
