"""Multi-step Pilot-Commit scheduling, written out from Algorithm 1.

Test infrastructure: reference for pc_sched_pilot / pc_sched_commit.

State: the replay buffer R (pilot survivors waiting for their commit pass,
Section 3.4 "Replay buffer for pilot survivors"), the set of prompts evicted
from the dataset pool D (Section 3.4 "Evicting solved prompts") and the step
counter t.

  pilot(uids, tags, p_hat)
      One sampling batch at the current step t (Algorithm 1, the Pilot /
      Filter / Evict / Buffer lines): every prompt is classified with the
      pilot filter B' = {q : p_lower <= p_hat <= p_upper}; prompts with
      p_hat >= p_solve leave the pool; the survivors B' are appended to R in
      batch order, stamped with t.  May be called more than once per step
      (a further sampling round, Section 5.4, when R cannot fill the batch).
  commit()
      The Commit lines: up to b_t prompts are taken out of R; then entries
      that could not be committed within the maximum delay d any more are
      dropped, and t <- t + 1.

Readings where the paper leaves the choice open (each also listed with the
other readings of this implementation):
  * order of selection from R ("sample prompt q from R"): the survivors of
    the current step first, in batch order (Section 3.4: only the EXCESS of
    a step goes to the buffer, and the buffer is drawn on when the current
    pilot yields too few); then buffered survivors, oldest step first, in
    their insertion order.
  * maximum delay d (Section 4.2, d = 4): an entry stamped t0 may be
    committed at steps t0 .. t0 + d.  Algorithm 1 drops "entries older than
    d steps" after the commit of step t and before t advances, so an entry
    is dropped there when t + 1 - t0 > d: it could only be used later than
    the delay allows.
  * threshold comparisons in fp32 on the fp32 p_hat, as in
    allocation.select_commit.

mean_rollouts_per_step: Section 5.4 prints the mean rollouts per step of
runs in which a fraction f of the steps needed a second sampling round; a
second round costs what a first one costs (Section 4.3 formula), so the
mean is cost * (1 + f).
"""
from __future__ import annotations

import numpy as np

HARD, KEEP, EASY = 0, 1, 2


class Scheduler:
    def __init__(self, p_lower, p_upper, p_solve, b_t, max_delay):
        if b_t <= 0 or max_delay < 0:
            raise ValueError("b_t must be positive and max_delay non-negative")
        self.lo, self.hi, self.so = np.float32(p_lower), np.float32(p_upper), np.float32(p_solve)
        self.b_t, self.d = int(b_t), int(max_delay)
        self.t = 0
        self.R = []                 # (uid, tag, t0), in insertion order
        self.evicted = set()
        self.rounds_this_step = 0
        self.stats = dict(pilot_batches=0, prompts_seen=0, buffered=0, committed=0, aged_out=0, evictions=0,
                          short_steps=0, multi_round_steps=0)

    def pilot(self, uids, tags, p_hat):
        """Returns (cls u8 [n], evict u8 [n], counts i32[4] = buffered, evicted, easy, hard)."""
        ph = np.asarray(p_hat, dtype=np.float32)
        n = len(ph)
        cls = np.empty(n, np.uint8)
        evict = np.zeros(n, np.uint8)
        for q in range(n):
            if ph[q] > self.hi:
                cls[q] = EASY
            elif ph[q] < self.lo:
                cls[q] = HARD
            else:
                cls[q] = KEEP
                self.R.append((int(uids[q]), int(tags[q]), self.t))
            if ph[q] >= self.so:
                evict[q] = 1
                self.evicted.add(int(uids[q]))
        counts = np.array([int(np.sum(cls == KEEP)), int(evict.sum()), int(np.sum(cls == EASY)),
                           int(np.sum(cls == HARD))], np.int32)
        self.rounds_this_step += 1
        self.stats["pilot_batches"] += 1
        self.stats["prompts_seen"] += n
        self.stats["buffered"] += int(counts[0])
        self.stats["evictions"] += int(counts[1])
        return cls, evict, counts

    def commit(self):
        """Returns ((uids, tags, ages) of the selected prompts, in selection order,
        (uids, tags) of the entries dropped for age, in buffer order)."""
        idx = [i for i, e in enumerate(self.R) if e[2] == self.t] + \
              [i for i, e in enumerate(self.R) if e[2] != self.t]      # insertion order = oldest step first
        idx = idx[:self.b_t]
        chosen = [self.R[i] for i in idx]
        rest = [e for i, e in enumerate(self.R) if i not in set(idx)]
        aged = [e for e in rest if self.t + 1 - e[2] > self.d]
        self.R = [e for e in rest if self.t + 1 - e[2] <= self.d]
        sel = (np.array([e[0] for e in chosen], np.int64), np.array([e[1] for e in chosen], np.int64),
               np.array([self.t - e[2] for e in chosen], np.int32))
        old = (np.array([e[0] for e in aged], np.int64), np.array([e[1] for e in aged], np.int64))
        self.stats["committed"] += len(chosen)
        self.stats["aged_out"] += len(aged)
        self.stats["short_steps"] += int(len(chosen) < self.b_t)
        self.stats["multi_round_steps"] += int(self.rounds_this_step > 1)
        self.rounds_this_step = 0
        self.t += 1
        return sel, old

    def is_evicted(self, uids):
        return np.array([int(u) in self.evicted for u in uids], np.uint8)

    def available(self):
        """Entries of R that the current step's commit could take."""
        return len(self.R)


def mean_rollouts_per_step(cost_per_round, second_round_fraction):
    """Mean rollouts per training step when a fraction of the steps runs a
    second sampling round of the same cost (Section 5.4)."""
    return cost_per_round * (1.0 + second_round_fraction)
