"""Reference forward pass of the decoder-only policy pi_theta(o_t | q, o_<t)
(Section 3.1): pre-norm transformer with RMSNorm, rotary positions
(rotate-half pairing), grouped-query causal attention and a SwiGLU FFN.

Test infrastructure: the HIP library's logits are compared with these.

Two implementations that must agree:
  forward_full    brute force: recompute the whole sequence, every position
  CachedDecoder   incremental: contiguous per-sequence K/V cache, no paging,
                  no prefix sharing
Everything is numpy in ``dtype`` (float64 by default).  Matrix products use
numpy's matmul; there is no blocking, fusion or reordering here.

Weight layout: every matrix is [out_features, in_features]; y = x @ W.T.
"""
from __future__ import annotations

import numpy as np


def _np(t, dtype):
    """torch tensor (fp32 or bf16) or ndarray -> ndarray of `dtype` (exact upcast)."""
    if isinstance(t, np.ndarray):
        return t.astype(dtype, copy=False)
    return t.detach().to("cpu").float().numpy().astype(dtype, copy=False)


class Shape:
    """The few model numbers the forward pass needs, taken from any object
    with the same attribute names."""

    def __init__(self, m):
        self.n_layers = int(m.n_layers)
        self.d_model = int(m.d_model)
        self.n_q_heads = int(m.n_q_heads)
        self.n_kv_heads = int(m.n_kv_heads)
        self.head_dim = int(m.head_dim)
        self.d_ff = int(m.d_ff)
        self.vocab = int(m.vocab)
        self.rms_eps = float(m.rms_eps)
        self.rope_theta = float(m.rope_theta)


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean_d(x^2) + eps) * gain, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope_cos_sin(positions, head_dim, theta):
    """Angles pos * theta^(-2i/hd), i = 0..hd/2-1, computed in float64."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)


def apply_rope(x, positions, theta):
    """x: [L, heads, hd]; pairs (i, i + hd/2) are rotated by the angle of
    pair i at the row's absolute position."""
    L, H, hd = x.shape
    cos, sin = rope_cos_sin(positions, hd, theta)
    cos = cos.astype(x.dtype)[:, None, :]
    sin = sin.astype(x.dtype)[:, None, :]
    x1, x2 = x[..., : hd // 2], x[..., hd // 2:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def gqa_attention(q, k, v, q_positions):
    """softmax(q k^T / sqrt(hd)) v with a causal mask.

    q: [Lq, hq, hd] at absolute positions q_positions; k, v: [Lk, hkv, hd]
    holding positions 0..Lk-1.  Query head j reads kv head j // (hq/hkv).
    """
    Lq, hq, hd = q.shape
    Lk, hkv, _ = k.shape
    rep = hq // hkv
    out = np.empty_like(q)
    scale = 1.0 / np.sqrt(np.array(hd, dtype=q.dtype))
    key_pos = np.arange(Lk)
    mask = key_pos[None, :] > np.asarray(q_positions)[:, None]          # [Lq, Lk]
    for j in range(hq):
        g = j // rep
        s = (q[:, j, :] @ k[:, g, :].T) * scale                         # [Lq, Lk]
        s = np.where(mask, -np.inf, s)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, j, :] = p @ v[:, g, :]
    return out


def _layer(shape, w, l, h, positions, k_prev, v_prev, dtype):
    """One decoder layer on rows h [L, d] at `positions`, attending to
    (k_prev, v_prev) [Lprev, hkv, hd] followed by the rows' own keys/values.
    Returns (h_out, k_all, v_all)."""
    s = shape
    a = rmsnorm(h, _np(w["attn_norm"][l], dtype), s.rms_eps)
    q = (a @ _np(w["wq"][l], dtype).T).reshape(-1, s.n_q_heads, s.head_dim)
    k = (a @ _np(w["wk"][l], dtype).T).reshape(-1, s.n_kv_heads, s.head_dim)
    v = (a @ _np(w["wv"][l], dtype).T).reshape(-1, s.n_kv_heads, s.head_dim)
    q = apply_rope(q, positions, s.rope_theta)
    k = apply_rope(k, positions, s.rope_theta)
    if k_prev is not None:
        k_all = np.concatenate([k_prev, k], axis=0)
        v_all = np.concatenate([v_prev, v], axis=0)
    else:
        k_all, v_all = k, v
    att = gqa_attention(q, k_all, v_all, positions).reshape(-1, s.n_q_heads * s.head_dim)
    h = h + att @ _np(w["wo"][l], dtype).T
    b = rmsnorm(h, _np(w["ffn_norm"][l], dtype), s.rms_eps)
    gate = b @ _np(w["w_gate"][l], dtype).T
    up = b @ _np(w["w_up"][l], dtype).T
    h = h + (silu(gate) * up) @ _np(w["w_down"][l], dtype).T
    return h, k_all, v_all


def _embed(w, tokens, dtype):
    """Rows of the embedding table (gathered first, then upcast)."""
    e = w["tok_embed"]
    if isinstance(e, np.ndarray):
        return e[tokens].astype(dtype)
    import torch
    return e[torch.as_tensor(np.asarray(tokens, dtype=np.int64))].float().numpy().astype(dtype)


def _logits(shape, w, h, dtype):
    return rmsnorm(h, _np(w["final_norm"], dtype), shape.rms_eps) @ _np(w["lm_head"], dtype).T


def forward_full(model, w, tokens, dtype=np.float64, rows=None, on_layer=None):
    """Brute force: logits for the whole sequence `tokens` [L] (or only for
    the positions listed in `rows`), recomputed from scratch.  `on_layer(l)`,
    if given, is called after each layer (progress reports of long runs)."""
    s = Shape(model)
    tokens = np.asarray(tokens, dtype=np.int64)
    pos = np.arange(len(tokens))
    h = _embed(w, tokens, dtype)
    for l in range(s.n_layers):
        h, _, _ = _layer(s, w, l, h, pos, None, None, dtype)
        if on_layer is not None:
            on_layer(l)
    if rows is not None:
        h = h[np.asarray(rows)]
    return _logits(s, w, h, dtype)


class CachedDecoder:
    """Incremental decoding of ONE sequence with a contiguous K/V cache."""

    def __init__(self, model, w, dtype=np.float64):
        self.s = Shape(model)
        self.w = w
        self.dtype = dtype
        self.k = [None] * self.s.n_layers
        self.v = [None] * self.s.n_layers
        self.length = 0

    def clone(self):
        c = CachedDecoder.__new__(CachedDecoder)
        c.s, c.w, c.dtype, c.length = self.s, self.w, self.dtype, self.length
        c.k = [None if x is None else x.copy() for x in self.k]
        c.v = [None if x is None else x.copy() for x in self.v]
        return c

    def extend(self, tokens, all_rows=False):
        """Feed `tokens` (positions length..length+n-1); returns the logits of
        the last fed row [V] (or of every fed row [n, V])."""
        tokens = np.atleast_1d(np.asarray(tokens, dtype=np.int64))
        pos = np.arange(self.length, self.length + len(tokens))
        h = _embed(self.w, tokens, self.dtype)
        for l in range(self.s.n_layers):
            h, self.k[l], self.v[l] = _layer(self.s, self.w, l, h, pos, self.k[l], self.v[l], self.dtype)
        self.length += len(tokens)
        if all_rows:
            return _logits(self.s, self.w, h, self.dtype)
        return _logits(self.s, self.w, h[-1:], self.dtype)[0]
