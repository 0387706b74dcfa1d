"""Plain CPU oracle for batched group rollout generation with Pilot-Commit
allocation.

TEST INFRASTRUCTURE ONLY.  This package is the slow, obviously-correct
reference the HIP library is checked against.  It shares no code with the
library, never imports it, and nothing on the product path may import it:
only the tests, the smoke check and the benchmark's CPU-baseline and
parity-sample legs do.

Modules
  philox      Philox4x32-10 counter-based generator (Salmon et al., SC'11)
  decoder     pre-norm GQA decoder forward: brute force and KV-cached
  sampler     temperature softmax + inverse-CDF sampling (Section 3.1 sampling), optionally
              restricted to the nucleus (top-p; Section 4.2 names the parameter)
  allocation  group statistics (Eq. 3), pilot filter / eviction / commit set
              (Section 3.3, Algorithm 1), the variance form of the filter for non-binary
              rewards (Section 3.3's remark on the extension; the rule is this implementation's reading),
              group-relative advantages, sampling cost (Section 4.3)
  scheduler   multi-step scheduling: replay buffer, maximum delay, eviction (Algorithm 1,
              Section 3.4)
  scoring     log-probability of a given completion under the policy (Section 3.1,
              the per-token factors of Eq. 2's ratio)
  rewards     the synthetic reward rules of the workloads (binary; one graded, four-valued)
  rollout     pilot pass -> select -> commit pass -> advantages, end to end

Pin status: every function here is pinned by tests/test_oracle_*.py against
closed forms, published known-answer vectors, invariants, brute force or an
independent library routine, except the end-to-end token sequences of
rollout.pilot_commit_step, for which no published values exist:
"parity unpinned" for those (their parts are each pinned).
"""
