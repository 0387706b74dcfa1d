"""Seeded synthetic inputs for batched group rollout generation.

This module only *draws inputs*: model shapes, random-init weights, uniform
prompts, per-prompt success probabilities and the uniforms a synthetic reward
consumes.  It holds none of the method's arithmetic (no transformer maths, no
sampler, no allocation rule), so both the CPU oracle's tests and the HIP
library's harness may import it; they share nothing else.

The shapes stand in for the model scales the paper trains (Section 4.1: 1.5B,
8B and 14B decoders) with its sampling settings (Section 4.2: temperature 1.0,
top_p 1.0, multi-thousand-token responses).  The paper's models, prompts and
verifier are replaced by random-init weights, uniform token prompts and
synthetic binary rewards.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np
import torch


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    dtype: str = "fp32"          # "fp32" or "bf16": storage type of the matrices
    tied_embeddings: bool = False

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def body_params(self) -> int:
        per_layer = (self.d_model * (self.q_dim + 2 * self.kv_dim)
                     + self.q_dim * self.d_model + 3 * self.d_model * self.d_ff)
        return self.n_layers * per_layer

    def lm_head_params(self) -> int:
        return self.vocab * self.d_model

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * self.elem_bytes()


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    n_prompts: int
    prompt_len: int
    n_pilot: int
    n_commit: int
    new_tokens: int
    temperature: float = 1.0
    top_p: float = 1.0           # nucleus sampling (1.0 = off: the paper's training setting, Section 4.2)
    reward: str = "last_even"    # "last_even" | "last_mod7" | "bernoulli" | "graded_mod7" (four-valued)
    filter: str = "binary"       # "binary": p_lower <= p_hat <= p_upper; "variance": on the pilot variance
    var_hard: float = 0.109375   # variance filter: threshold while the mean is <= mean_pivot (0.125 * 0.875)
    var_easy: float = 0.1875     #                  threshold beyond it (0.75 * 0.25)
    mean_pivot: float = 0.5
    eos: bool = False            # per-sequence early stop at a seeded EOS id
    p_lower: float = 0.125       # Section 4.2 thresholds
    p_upper: float = 0.75
    p_solve: float = 1.0
    b_t: int = 0                 # cap on committed prompts; 0 = no cap
    seed_weights: int = 1
    seed_prompts: int = 2
    seed_sampler: int = 3
    seed_eos: int = 4
    seed_reward: int = 5


_QWEN15 = ModelShape(28, 1536, 12, 2, 128, 8960, 151936, 1e-6, 1.0e6, "bf16", True)
_QWEN8 = ModelShape(36, 4096, 32, 8, 128, 12288, 151936, 1e-6, 1.0e6, "bf16", False)
_QWEN14 = ModelShape(40, 5120, 40, 8, 128, 17408, 151936, 1e-6, 1.0e6, "bf16", False)

WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", ModelShape(2, 128, 4, 2, 32, 384, 512, 1e-6, 1.0e4, "fp32", False),
                   8, 32, 4, 4, 16, reward="last_even"),
    "C2": Workload("C2", _QWEN15, 64, 256, 4, 4, 1024, reward="last_mod7"),
    "C3": Workload("C3", _QWEN15, 128, 512, 8, 8, 2048, reward="last_mod7", eos=True),
    "C4": Workload("C4", _QWEN8, 64, 512, 4, 12, 2048, reward="bernoulli"),
    "C5": Workload("C5", _QWEN14, 32, 1024, 4, 12, 4096, reward="bernoulli", eos=True),
    # the 1.5B stress shape with the paper's evaluation sampling (Section 4.2: temperature 0.7; top-p is an
    # addition here: 0.95) and a four-valued reward selected on by the variance filter
    "C3E": Workload("C3E", _QWEN15, 128, 512, 8, 8, 2048, temperature=0.7, top_p=0.95, reward="graded_mod7",
                    filter="variance", var_hard=0.02, var_easy=0.05, eos=True),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller slices for tests)."""
    model_kw = {k: v for k, v in kw.items() if k in ModelShape.__dataclass_fields__}
    wl_kw = {k: v for k, v in kw.items() if k not in model_kw}
    if model_kw:
        wl_kw["model"] = replace(w.model, **model_kw)
    return replace(w, **wl_kw)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------

MATRIX_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def _matrix_shapes(m: ModelShape) -> Dict[str, tuple]:
    # all matrices are stored row-major as [out_features, in_features]
    return {
        "wq": (m.q_dim, m.d_model), "wk": (m.kv_dim, m.d_model), "wv": (m.kv_dim, m.d_model),
        "wo": (m.d_model, m.q_dim),
        "w_gate": (m.d_ff, m.d_model), "w_up": (m.d_ff, m.d_model), "w_down": (m.d_model, m.d_ff),
    }


def make_weights(m: ModelShape, seed: int, device: str = "cpu", std: float = 0.02) -> dict:
    """Random-init decoder weights: matrices and embeddings ~ N(0, std), norm
    gains = 1, no biases.  Matrices are rounded to the model's storage dtype
    here, once, so that every consumer sees the same bytes.  Norm gains are
    always fp32.  With ``device="cuda"`` the draw happens on the GPU (fast for
    the multi-billion-parameter shapes); the values then differ from the CPU
    draw of the same seed, which is fine as long as one draw feeds both sides.
    """
    tdt = torch.float32 if m.dtype == "fp32" else torch.bfloat16
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))

    def normal(*shape):
        return (torch.randn(*shape, generator=gen, device=device, dtype=torch.float32) * std).to(tdt)

    w: dict = {"tok_embed": normal(m.vocab, m.d_model)}
    w["lm_head"] = w["tok_embed"] if m.tied_embeddings else normal(m.vocab, m.d_model)
    w["final_norm"] = torch.ones(m.d_model, dtype=torch.float32, device=device)
    shapes = _matrix_shapes(m)
    for name in MATRIX_NAMES:
        w[name] = []
    w["attn_norm"], w["ffn_norm"] = [], []
    for _ in range(m.n_layers):
        w["attn_norm"].append(torch.ones(m.d_model, dtype=torch.float32, device=device))
        w["ffn_norm"].append(torch.ones(m.d_model, dtype=torch.float32, device=device))
        for name in MATRIX_NAMES:
            w[name].append(normal(*shapes[name]))
    return w


def perturb_norm_gains(w: dict, seed: int, spread: float = 0.25) -> dict:
    """Replace the all-ones norm gains by 1 + U(-spread, spread) (test-only: a
    gain of exactly 1 would hide a dropped or misplaced gain multiply)."""
    gen = torch.Generator().manual_seed(int(seed))

    def g(t):
        return (1.0 + spread * (2.0 * torch.rand(t.shape, generator=gen) - 1.0)).to(t.dtype).to(t.device)

    out = dict(w)
    out["final_norm"] = g(w["final_norm"])
    out["attn_norm"] = [g(t) for t in w["attn_norm"]]
    out["ffn_norm"] = [g(t) for t in w["ffn_norm"]]
    return out


def weights_to(w: dict, device: str) -> dict:
    out = {}
    moved: dict = {}
    for k, v in w.items():
        if isinstance(v, list):
            out[k] = [t.to(device) for t in v]
        else:
            if id(v) not in moved:          # keep tied tensors tied
                moved[id(v)] = v.to(device)
            out[k] = moved[id(v)]
    return out


# --------------------------------------------------------------------------
# prompts, EOS id, reward inputs
# --------------------------------------------------------------------------

def make_prompts(n_prompts: int, prompt_len: int, vocab: int, seed: int) -> np.ndarray:
    """[P, Lp] int32 token ids, uniform over the vocabulary."""
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    return rng.integers(0, vocab, size=(n_prompts, prompt_len), dtype=np.int32)


def make_ragged_prompts(lens: List[int], vocab: int, seed: int):
    """Packed prompts of unequal length: (tokens[sum lens], cu_lens[P+1])."""
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    toks = rng.integers(0, vocab, size=int(cu[-1]), dtype=np.int32)
    return toks, cu


def make_eos_id(vocab: int, seed: int) -> int:
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    return int(rng.integers(0, vocab))


def make_prompt_uids(n_prompts: int, first: int = 0) -> np.ndarray:
    return np.arange(first, first + n_prompts, dtype=np.int64)


def make_success_probs(n_prompts: int, seed: int) -> np.ndarray:
    """Per-prompt success probability p_q ~ Beta(1/2, 1/2), drawn by inverse
    CDF: p = sin^2(pi v / 2), v uniform.  An input distribution only; the
    reward rule that consumes it lives with each implementation."""
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    v = rng.random(n_prompts)
    return (np.sin(0.5 * np.pi * v) ** 2).astype(np.float32)


def make_reward_uniforms(n_prompts: int, n_rollouts: int, seed: int) -> np.ndarray:
    """[P, n_rollouts] fp32 uniforms in [0,1) consumed by the Bernoulli reward."""
    rng = np.random.Generator(np.random.PCG64(int(seed) + 7919))
    return rng.random((n_prompts, n_rollouts), dtype=np.float32)


def make_binary_rewards(group_sizes: List[int], seed: int, p: Optional[np.ndarray] = None):
    """Packed binary rewards for groups of the given sizes, plus offsets."""
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    off = np.zeros(len(group_sizes) + 1, dtype=np.int32)
    off[1:] = np.cumsum(np.asarray(group_sizes, dtype=np.int64))
    if p is None:
        p = rng.random(len(group_sizes))
    r = np.concatenate([(rng.random(g) < p[i]).astype(np.float32) for i, g in enumerate(group_sizes)]
                       + [np.zeros(0, np.float32)])
    return r, off
