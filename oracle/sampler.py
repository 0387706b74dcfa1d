"""Sampling one token o_t ~ pi_theta(. | q, o_<t) at temperature T with
top_p = 1 (Section 3.1; Section 4.2 sampling settings): temperature softmax
followed by inverse-CDF selection with a given uniform.

Test infrastructure: the definition the HIP sampler's tokens are checked
against.  The CDF is accumulated in float64 in index order; that order is
the definition of which token a uniform selects.
"""
from __future__ import annotations

import math

import numpy as np


def sample_token(logits, temperature: float, u: float, eos_id: int = -1, eos_logit_bias: float = 0.0):
    """logits: [V] (any float dtype, taken as fp32 values); u in (0,1).

    x_j = logit_j / T (+ bias on the EOS id); w_j = exp(x_j - max x);
    Z = sum w; token = the smallest i whose inclusive prefix sum exceeds u*Z,
    or, if rounding leaves none, the largest i with w_i > 0.
    Returns (token, logprob) with logprob = x_tok - max x - ln Z.
    """
    x = np.asarray(logits, dtype=np.float32).astype(np.float64) / float(temperature)
    if eos_id >= 0 and eos_logit_bias != 0.0:
        x = x.copy()
        x[eos_id] += float(eos_logit_bias)
    m = x.max()
    w = np.exp(x - m)
    cdf = np.cumsum(w)                      # sequential, index order, float64
    Z = cdf[-1]
    target = float(u) * Z
    hit = np.nonzero(cdf > target)[0]
    if len(hit):
        tok = int(hit[0])
    else:
        tok = int(np.nonzero(w > 0)[0][-1])
    logprob = float(x[tok] - m - math.log(Z))
    return tok, logprob


def softmax_probs(logits, temperature: float = 1.0):
    x = np.asarray(logits, dtype=np.float64) / float(temperature)
    w = np.exp(x - x.max())
    return w / w.sum()
