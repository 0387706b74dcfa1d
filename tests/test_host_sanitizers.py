"""The library's host-side C++ (the multi-step scheduler, the KV-cache
bookkeeping and the kernels' index maps: real sources, no copies) built for
the CPU with the address and undefined-behaviour sanitizers and driven without
a GPU:

  * the scheduler replays a synthetic multi-epoch training run (drifting
    success rates, second sampling rounds, age-outs, evictions) and every
    output is compared with the oracle's Algorithm 1 loop;
  * the bookkeeping runs thousands of random prefill / fork / decode /
    release operations with all of its invariants checked after each.

Any out-of-bounds access, use after free, leak or undefined operation makes
the sanitized program exit non-zero."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import scheduler as osched

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host", "host_checks.hip")


@pytest.fixture(scope="module")
def host_checks(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc to build the sanitized host program with")
    exe = str(tmp_path_factory.mktemp("host") / "host_checks")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined", SRC, "-o", exe]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout
    return exe


def _run(exe, args, stdin=""):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe] + args, input=stdin, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env,
                       timeout=300)
    assert p.returncode == 0, "exit %d\n%s\n%s" % (p.returncode, p.stdout[-2000:], p.stderr[-4000:])
    assert "ERROR: AddressSanitizer" not in p.stderr and "runtime error" not in p.stderr, p.stderr[-4000:]
    return p.stdout


def test_index_maps_exhaustively(host_checks):
    """The kernels' index arithmetic (csrc/index_maps.h, the same header the kernels include): the operand-fragment
    cache layout and the GEMM's tile order, checked over every geometry the library accepts."""
    out = _run(host_checks, ["maps"])
    assert out.startswith("maps ok")


def test_kv_bookkeeping_under_sanitizers(host_checks):
    out = _run(host_checks, ["book", "6000"])
    assert out.startswith("book ok: 6000 operations")
    forks = int(out.split(" forks")[0].split()[-1])
    assert forks > 200


@pytest.mark.parametrize("b_t,d,s_factor,n_pilot", [(16, 4, 3, 8), (5, 2, 1, 4), (8, 0, 3, 4)])
def test_scheduler_under_sanitizers_follows_the_oracle(host_checks, b_t, d, s_factor, n_pilot):
    lo, hi, solve = 0.125, 0.75, 1.0
    rng = np.random.default_rng(b_t * 10 + d)
    n_prompts = 40 * b_t
    p_q = np.sin(0.5 * np.pi * rng.random(n_prompts)) ** 2
    uids = np.arange(n_prompts, dtype=np.int64) * 7 + 3
    want = osched.Scheduler(lo, hi, solve, b_t, d)
    trace = ["S %r %r %r %d %d" % (lo, hi, solve, b_t, d)]
    expect = []
    steps = 0
    for _ in range(3):
        ev = want.is_evicted(uids)
        trace.append("E %d %s" % (n_prompts, " ".join(map(str, uids.tolist()))))
        expect.append("E " + " ".join(str(int(x)) for x in ev))
        pool = rng.permutation(np.nonzero(ev == 0)[0])
        pos = 0
        while pos < len(pool):
            rounds = 0
            while pos < len(pool) and rounds < 2:
                batch = pool[pos:pos + s_factor * b_t]
                pos += len(batch)
                p_hat = (rng.binomial(n_pilot, p_q[batch]) / np.float32(n_pilot)).astype(np.float32)
                tags = (batch.astype(np.int64) << 20) + steps
                cls, evict, counts = want.pilot(uids[batch], tags, p_hat)
                trace.append("P %d %s" % (len(batch), " ".join("%d %d %r" % (u, t, float(p))
                                                                for u, t, p in zip(uids[batch], tags, p_hat))))
                expect.append("P " + " ".join("%d%d" % (c, e) for c, e in zip(cls, evict)) +
                              " | %d %d %d %d" % tuple(int(x) for x in counts))
                rounds += 1
                if want.available() >= b_t:
                    break
            (su, st, sa), (au, at) = want.commit()
            trace.append("C")
            expect.append(("C " + " ".join("%d:%d:%d" % (u, t, a) for u, t, a in zip(su, st, sa))).rstrip() + " |" +
                          "".join(" %d:%d" % (u, t) for u, t in zip(au, at)))
            steps += 1
            p_q = np.minimum(1.0, p_q + 0.004)
    trace.append("T")
    out = _run(host_checks, ["sched"], "\n".join(trace) + "\n").strip().splitlines()
    assert len(out) == len(expect) + 1
    for i, (g, w) in enumerate(zip(out, expect)):
        assert g.strip() == w.strip(), "line %d" % i
    stats = [int(x) for x in out[-1].split()[1:]]
    names = ("step", "buffered_now", "pilot_batches", "prompts_seen", "buffered", "committed", "aged_out", "evictions",
             "short_steps", "multi_round_steps")
    got = dict(zip(names, stats))
    assert got["step"] == want.t == steps and got["buffered_now"] == want.available()
    for k, v in want.stats.items():
        assert got[k] == v, k
    assert steps > 20 and got["committed"] > 0
