"""Synthetic binary rewards R(q, o) in {0, 1} (Section 3.3) standing in for
the paper's math verifier.  Test infrastructure.

  last_even   1 iff the last generated token id is even
  last_mod7   1 iff (last generated token id mod 7) == (prompt uid mod 7)
  bernoulli   1 iff u < p_q, with p_q the prompt's success probability and u
              a supplied uniform
  graded_mod7 a four-valued reward in {0, 1/3, 2/3, 1} (a stand-in for rewards
              that are not binary, Section 7): 1 - d/3 with d the distance on
              the circle of residues mod 7 between the last generated token id
              and the prompt uid
The "last generated token" of a sequence stopped by EOS is the EOS itself.
"""
from __future__ import annotations

import numpy as np


def last_token(tokens_row, length):
    return int(tokens_row[int(length) - 1])


def reward(rule, last_tok=None, prompt_uid=None, p_q=None, u=None) -> float:
    if rule == "last_even":
        return 1.0 if last_tok % 2 == 0 else 0.0
    if rule == "last_mod7":
        return 1.0 if last_tok % 7 == int(prompt_uid) % 7 else 0.0
    if rule == "bernoulli":
        return 1.0 if np.float32(u) < np.float32(p_q) else 0.0
    if rule == "graded_mod7":
        d = (last_tok - int(prompt_uid)) % 7
        d = min(d, 7 - d)                      # 0 .. 3
        return float(np.float32(3 - d) / np.float32(3.0))
    raise ValueError(rule)
