"""Teacher-forced scoring: the policy's log-probability of a given completion.

Test infrastructure: reference for pc_score.

Section 3.1 writes a rollout's probability as the product over its tokens of
pi_theta(o_t | q, o_<t); the objective's importance ratio (Eq. 2) is a ratio
of exactly these per-token probabilities under two policies.  For a sequence
(prompt q followed by completion o) this returns

    log pi_theta(o_t | q, o_<t)  =  x_t[o_t] - max x_t - log sum_j exp(x_t[j] - max x_t),
    x_t = logits at the position before o_t, divided by the temperature,

for every completion token, the logits coming from the brute-force forward
of the decoder oracle (float64).
"""
from __future__ import annotations

import numpy as np

from . import decoder


def log_softmax_at(logits, temperature, token):
    """log softmax(logits / temperature)[token]; sums in float64, index order."""
    x = np.asarray(logits, dtype=np.float64) / float(temperature)
    m = x.max()
    z = 0.0
    for v in x:
        z += np.exp(v - m)
    return float(x[token] - m - np.log(z))


def score(model, w, tokens, prompt_len, temperature=1.0):
    """tokens: the whole sequence (prompt + completion); prompt_len >= 1.
    Returns float64 [len(tokens) - prompt_len]: log-probability of each
    completion token given everything before it."""
    tokens = np.asarray(tokens)
    n = len(tokens)
    if not 1 <= prompt_len <= n:
        raise ValueError("prompt_len must lie in 1 .. len(tokens)")
    if prompt_len == n:
        return np.zeros(0, np.float64)
    rows = np.arange(prompt_len - 1, n - 1)
    logits = decoder.forward_full(model, w, tokens[:-1], rows=rows)
    return np.array([log_softmax_at(logits[i], temperature, int(tokens[prompt_len + i])) for i in range(len(rows))])
