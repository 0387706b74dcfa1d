"""Pins for oracle.decoder: an independent implementation on torch's library
ops, brute force vs cached, closed-form degenerate cases and invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads
from oracle import decoder

TINY = workloads.WORKLOADS["C1"].model


def _weights(model=TINY, seed=11, gains=True):
    w = workloads.make_weights(model, seed)
    if gains:
        w = workloads.perturb_norm_gains(w, seed + 1)
    return w


def torch_library_forward(m, w, tokens):
    """The same architecture on torch's own operators, with RoPE written as a
    complex rotation of the pair (x_i, x_{i+hd/2})."""
    tok = torch.as_tensor(np.asarray(tokens, dtype=np.int64))
    L = len(tok)
    h = w["tok_embed"].double()[tok]
    pos = torch.arange(L, dtype=torch.float64)
    inv = m.rope_theta ** (-torch.arange(0, m.head_dim, 2, dtype=torch.float64) / m.head_dim)
    rot = torch.polar(torch.ones(L, m.head_dim // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

    def rope(x):  # [L, H, hd]
        z = torch.complex(x[..., : m.head_dim // 2], x[..., m.head_dim // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(m.n_layers):
        a = F.rms_norm(h, (m.d_model,), w["attn_norm"][l].double(), m.rms_eps)
        q = rope(F.linear(a, w["wq"][l].double()).view(L, m.n_q_heads, m.head_dim))
        k = rope(F.linear(a, w["wk"][l].double()).view(L, m.n_kv_heads, m.head_dim))
        v = F.linear(a, w["wv"][l].double()).view(L, m.n_kv_heads, m.head_dim)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)
        o = o[0].transpose(0, 1).reshape(L, m.q_dim)
        h = h + F.linear(o, w["wo"][l].double())
        b = F.rms_norm(h, (m.d_model,), w["ffn_norm"][l].double(), m.rms_eps)
        h = h + F.linear(F.silu(F.linear(b, w["w_gate"][l].double())) * F.linear(b, w["w_up"][l].double()),
                         w["w_down"][l].double())
    return F.linear(F.rms_norm(h, (m.d_model,), w["final_norm"].double(), m.rms_eps), w["lm_head"].double()).numpy()


@pytest.mark.parametrize("shape_kw", [
    {},                                                      # C1: 4 q heads on 2 kv heads
    {"n_q_heads": 6, "n_kv_heads": 2, "d_model": 96},        # ratio 3
    {"n_q_heads": 4, "n_kv_heads": 4},                       # plain multi-head attention
    {"n_q_heads": 4, "n_kv_heads": 1},                       # multi-query
])
def test_matches_torch_library_ops(shape_kw):
    m = workloads.scaled(workloads.WORKLOADS["C1"], **shape_kw).model
    w = _weights(m, std_seed := 5)
    toks = workloads.make_prompts(1, 23, m.vocab, 9)[0]
    got = decoder.forward_full(m, w, toks)
    want = torch_library_forward(m, w, toks)
    assert np.abs(got - want).max() < 1e-10
    # logits must not be degenerate, or the comparison says nothing
    assert np.abs(want).max() > 1e-2


def test_larger_std_exercises_softmax():
    # N(0, 0.02) weights give nearly flat attention; a larger spread makes the
    # softmax, the causal mask and the 1/sqrt(hd) scale matter
    m = TINY
    w = workloads.perturb_norm_gains(workloads.make_weights(m, 21, std=0.3), 22)
    toks = workloads.make_prompts(1, 17, m.vocab, 23)[0]
    got = decoder.forward_full(m, w, toks)
    want = torch_library_forward(m, w, toks)
    assert np.abs(got - want).max() < 1e-8 * max(1.0, np.abs(want).max())


def test_cached_equals_brute_force():
    m, w = TINY, _weights()
    toks = workloads.make_prompts(1, 20, m.vocab, 3)[0]
    full = decoder.forward_full(m, w, toks)
    dec = decoder.CachedDecoder(m, w)
    first = dec.extend(toks[:12])
    assert np.abs(first - full[11]).max() < 1e-12
    for t in range(12, 20):
        row = dec.extend([toks[t]])
        assert np.abs(row - full[t]).max() < 1e-12
    # fp32 arithmetic: the two routes agree to fp32 rounding
    full32 = decoder.forward_full(m, w, toks, dtype=np.float32)
    dec32 = decoder.CachedDecoder(m, w, np.float32)
    dec32.extend(toks[:12])
    row = dec32.extend(toks[12:13])
    assert np.abs(row - full32[12]).max() < 1e-5
    assert np.abs(full32 - full).max() < 1e-4


def test_causality():
    m, w = TINY, _weights()
    a = workloads.make_prompts(1, 16, m.vocab, 4)[0]
    b = a.copy()
    b[10:] = (b[10:] + 1) % m.vocab
    la, lb = decoder.forward_full(m, w, a), decoder.forward_full(m, w, b)
    assert np.abs(la[:10] - lb[:10]).max() == 0.0
    assert np.abs(la[10:] - lb[10:]).max() > 1e-6


def test_clone_shares_prefix_exactly():
    # continuing from a copy of the prompt's state equals running prompt +
    # continuation privately
    m, w = TINY, _weights()
    prompt = workloads.make_prompts(1, 9, m.vocab, 5)[0]
    base = decoder.CachedDecoder(m, w)
    base.extend(prompt)
    for cont in ([3, 4, 5], [500, 1]):
        c = base.clone()
        for t in cont:
            got = c.extend([t])
        want = decoder.forward_full(m, w, np.concatenate([prompt, cont]))[-1]
        assert np.abs(got - want).max() < 1e-12
    assert base.length == 9


def test_zero_output_projections_closed_form():
    # W_o = W_down = 0 removes both residual branches:
    # logits = RMSNorm(E[tok]) W_lm^T
    m = TINY
    w = _weights()
    w = dict(w)
    w["wo"] = [torch.zeros_like(t) for t in w["wo"]]
    w["w_down"] = [torch.zeros_like(t) for t in w["w_down"]]
    toks = workloads.make_prompts(1, 7, m.vocab, 6)[0]
    got = decoder.forward_full(m, w, toks)
    e = w["tok_embed"].double().numpy()[toks]
    n = e / np.sqrt((e * e).mean(-1, keepdims=True) + m.rms_eps) * w["final_norm"].double().numpy()
    want = n @ w["lm_head"].double().numpy().T
    assert np.abs(got - want).max() < 1e-12


def test_rmsnorm_definition():
    x = np.array([[3.0, 4.0, 0.0, 0.0]])
    g = np.array([1.0, 2.0, 3.0, 4.0])
    # mean square = 25/4
    want = x / math.sqrt(25.0 / 4.0 + 0.5) * g
    assert np.allclose(decoder.rmsnorm(x, g, 0.5), want, rtol=0, atol=1e-15)


def test_rope_properties():
    hd, theta = 32, 10000.0
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, hd))
    # position 0 is the identity
    assert np.array_equal(decoder.apply_rope(x[:1], [0], theta), x[:1])
    # rotations preserve the norm of every (i, i+hd/2) pair
    y = decoder.apply_rope(x, [0, 1, 2, 50, 1000], theta)
    assert np.allclose(x[..., :16] ** 2 + x[..., 16:] ** 2, y[..., :16] ** 2 + y[..., 16:] ** 2)
    # pair 0 turns by exactly `pos` radians, the last pair by pos * theta^(-(hd-2)/hd)
    e = np.zeros((1, 1, hd))
    e[0, 0, 0] = 1.0
    r = decoder.apply_rope(e, [2], theta)
    assert np.allclose([r[0, 0, 0], r[0, 0, 16]], [math.cos(2.0), math.sin(2.0)])
    e = np.zeros((1, 1, hd))
    e[0, 0, 15] = 1.0
    r = decoder.apply_rope(e, [7], theta)
    ang = 7.0 * theta ** (-30.0 / 32.0)
    assert np.allclose([r[0, 0, 15], r[0, 0, 31]], [math.cos(ang), math.sin(ang)])
    # q.k after rotation depends only on the relative position
    q, k = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    d1 = (decoder.apply_rope(q, [9], theta) * decoder.apply_rope(k, [4], theta)).sum()
    d2 = (decoder.apply_rope(q, [105], theta) * decoder.apply_rope(k, [100], theta)).sum()
    assert abs(d1 - d2) < 1e-9


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    hq, hkv, hd = 4, 2, 8
    # a single key: the output is its value, for the right kv head
    q = rng.standard_normal((1, hq, hd))
    k = rng.standard_normal((1, hkv, hd))
    v = rng.standard_normal((1, hkv, hd))
    o = decoder.gqa_attention(q, k, v, [0])
    for j in range(hq):
        assert np.allclose(o[0, j], v[0, j // 2])
    # zero queries: uniform average over the visible keys only
    L = 6
    k = rng.standard_normal((L, hkv, hd))
    v = rng.standard_normal((L, hkv, hd))
    o = decoder.gqa_attention(np.zeros((L, hq, hd)), k, v, np.arange(L))
    for i in range(L):
        assert np.allclose(o[i, 3], v[: i + 1, 1].mean(0))
    # two keys, closed form with the 1/sqrt(hd) scale
    q = np.zeros((1, 1, hd)); q[0, 0, 0] = 2.0
    k = np.zeros((2, 1, hd)); k[1, 0, 0] = 3.0
    v = np.zeros((2, 1, hd)); v[0, 0, 0] = 1.0; v[1, 0, 1] = 1.0
    o = decoder.gqa_attention(q, k, v, [1])
    p1 = 1.0 / (1.0 + math.exp(-6.0 / math.sqrt(hd)))
    assert np.allclose(o[0, 0, :2], [1 - p1, p1])


def test_bf16_weights_upcast_exactly():
    m = workloads.scaled(workloads.WORKLOADS["C1"], dtype="bf16").model
    w = workloads.make_weights(m, 3)
    assert w["wq"][0].dtype == torch.bfloat16
    toks = workloads.make_prompts(1, 5, m.vocab, 1)[0]
    got = decoder.forward_full(m, w, toks)
    w64 = {k: ([t.double().numpy() for t in v] if isinstance(v, list) else v.double().numpy()) for k, v in w.items()}
    want = decoder.forward_full(m, w64, toks)
    assert np.array_equal(got, want)
