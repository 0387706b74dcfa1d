"""Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
easy as 1, 2, 3", SC'11), written out from the published round function.

Test infrastructure: reference for the sampler's random stream.

One round maps a counter (c0,c1,c2,c3) and key (k0,k1) to
  (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
with M0 = 0xD2511F53, M1 = 0xCD9E8D57; the key is bumped by the Weyl
constants (0x9E3779B9, 0xBB67AE85) between rounds; ten rounds in all.
"""
from __future__ import annotations

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF

DOMAIN_TOKEN = 0


def philox4x32_10(counter, key):
    """counter: 4 uint32, key: 2 uint32 -> 4 uint32 (python ints)."""
    c0, c1, c2, c3 = (int(x) & MASK for x in counter)
    k0, k1 = (int(x) & MASK for x in key)
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK, p1 & MASK, ((p0 >> 32) ^ c3 ^ k1) & MASK, p0 & MASK
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def uniform_from_bits(x: int) -> float:
    """Top 23 bits -> u = (x>>9 + 0.5) * 2^-23: strictly inside (0,1) and exact
    in fp32 (23 bits plus the half fill the 24-bit significand)."""
    return ((int(x) >> 9) + 0.5) * (1.0 / 8388608.0)


def sampling_uniform(seed: int, seq_uid: int, step: int, domain: int = DOMAIN_TOKEN) -> float:
    """The uniform that decides token `step` of the sequence `seq_uid`.

    key = (seed low word, seed high word); counter = (step, uid low word,
    uid high word, domain).  The stream depends on neither batch position
    nor the order in which sequences are compacted."""
    key = (seed & MASK, (seed >> 32) & MASK)
    ctr = (step & MASK, seq_uid & MASK, (seq_uid >> 32) & MASK, domain & MASK)
    return uniform_from_bits(philox4x32_10(ctr, key)[0])


def seq_uid(prompt_uid: int, rollout_index: int) -> int:
    """Sequence uid = prompt uid * 2^16 + rollout index; pilot rollouts take
    indices [0, n_pilot), commit rollouts [n_pilot, n_pilot + n_commit)."""
    return (int(prompt_uid) << 16) + int(rollout_index)
