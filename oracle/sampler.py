"""Sampling one token o_t ~ pi_theta(. | q, o_<t) at temperature T
(Section 3.1; Section 4.2 sampling settings: temperature 1.0 and top_p = 1.0
for training, temperature 0.7 for evaluation): temperature softmax, optional
nucleus (top-p) truncation, inverse-CDF selection with a given uniform.

Test infrastructure: the definition the HIP sampler's tokens are checked
against.  The CDF is accumulated in float64 in index order; that order is
the definition of which token a uniform selects.

Nucleus truncation (top_p < 1; the paper names the parameter and fixes it to
1.0 for training, it does not define it: this is the usual definition): the
tokens are taken in order of decreasing probability, equal probabilities in
order of increasing id, until their cumulative weight (float64, in that order)
reaches top_p * Z; only those tokens keep their weight.  The inverse CDF then
runs over the kept tokens in id order, renormalised to their own mass.
"""
from __future__ import annotations

import math

import numpy as np


def nucleus(w, top_p: float):
    """Boolean mask of the tokens kept by top-p truncation of the (unnormalised,
    non-negative) weights w: the shortest prefix of the tokens sorted by
    decreasing weight (ties: increasing id) whose cumulative weight reaches
    top_p * sum(w).  top_p is taken at its fp32 value (the library's argument
    type)."""
    w = np.asarray(w, dtype=np.float64)
    order = np.argsort(-w, kind="stable")   # decreasing weight; stable: equal weights keep id order
    c = np.cumsum(w[order])                 # sequential, in that order, float64
    target = float(np.float32(top_p)) * float(np.cumsum(w)[-1])
    reached = np.nonzero(c >= target)[0]
    k = int(reached[0]) if len(reached) else len(w) - 1
    keep = np.zeros(len(w), dtype=bool)
    keep[order[:k + 1]] = True
    return keep


def sample_token(logits, temperature: float, u: float, eos_id: int = -1, eos_logit_bias: float = 0.0,
                 top_p: float = 1.0):
    """logits: [V] (any float dtype, taken as fp32 values); u in (0,1).

    x_j = logit_j / T (+ bias on the EOS id); w_j = exp(x_j - max x);
    with top_p < 1 the weights outside the nucleus are set to 0;
    Z = sum w; token = the smallest i whose inclusive prefix sum exceeds u*Z,
    or, if rounding leaves none, the largest i with w_i > 0.
    Returns (token, logprob) with logprob = x_tok - max x - ln Z (the
    log-probability under the distribution sampled from).
    """
    x = np.asarray(logits, dtype=np.float32).astype(np.float64) / float(temperature)
    if eos_id >= 0 and eos_logit_bias != 0.0:
        x = x.copy()
        x[eos_id] += float(eos_logit_bias)
    m = x.max()
    w = np.exp(x - m)
    if top_p < 1.0:
        w = np.where(nucleus(w, top_p), w, 0.0)
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
