"""GPU parity: pc_group_stats / pc_select_commit / pc_advantages against the
oracle, element by element.  Integer, byte and index outputs are bit-exact;
fp32 statistics are bit-exact for binary rewards (both sides form them in
double and round once) and within 1 ulp otherwise."""
import numpy as np
import pytest
import torch

import workloads
from oracle import allocation as al
from gpu_util import say

pytestmark = pytest.mark.gpu


def _stats(r, off):
    import paper_2605_26606_amd as pc
    P = len(off) - 1
    d = "cuda"
    rd, od = torch.from_numpy(r).to(d), torch.from_numpy(off).to(d)
    n_pos = torch.full((max(P, 1),), -7, dtype=torch.int32, device=d)
    n_tot = torch.full((max(P, 1),), -7, dtype=torch.int32, device=d)
    mean = torch.full((max(P, 1),), -7.0, device=d)
    var = torch.full((max(P, 1),), -7.0, device=d)
    pc.pc_group_stats(rd, od, n_pos, n_tot, mean, var)
    torch.cuda.synchronize()
    return n_pos[:P].cpu().numpy(), n_tot[:P].cpu().numpy(), mean[:P].cpu().numpy(), var[:P].cpu().numpy()


@pytest.mark.parametrize("sizes", [[4] * 64, [8] * 128, [16] * 37, [32] * 5, [1], [3, 0, 7, 1, 16, 0, 128, 2]])
def test_group_stats_binary(sizes):
    say("group_stats binary sizes=%s..." % sizes[:4])
    r, off = workloads.make_binary_rewards(sizes, seed=len(sizes))
    got = _stats(r, off)
    want = al.group_stats(r, off)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


def test_group_stats_float_rewards_and_all_k():
    rng = np.random.default_rng(0)
    sizes = [5, 9, 1, 64, 1000]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = rng.standard_normal(off[-1]).astype(np.float32)
    got, want = _stats(r, off), al.group_stats(r, off)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    assert np.array_equal(got[2], want[2]) and np.array_equal(got[3], want[3])
    for n in (4, 8, 16, 32):            # every k for the paper's pilot sizes
        r = np.concatenate([np.r_[np.ones(k), np.zeros(n - k)] for k in range(n + 1)]).astype(np.float32)
        off = (np.arange(n + 2) * n).astype(np.int32)
        got, want = _stats(r, off), al.group_stats(r, off)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)
        assert got[3][0] == 0.0 and got[3][n] == 0.0


def _select(ph, lo, hi, so, b_t):
    import paper_2605_26606_amd as pc
    d = "cuda"
    P = len(ph)
    cls = torch.full((max(P, 1),), 9, dtype=torch.uint8, device=d)
    ev = torch.full((max(P, 1),), 9, dtype=torch.uint8, device=d)
    ci = torch.full((max(P, 1),), -1, dtype=torch.int32, device=d)
    si = torch.full((max(P, 1),), -1, dtype=torch.int32, device=d)
    cnt = torch.full((4,), -1, dtype=torch.int32, device=d)
    pc.pc_select_commit(torch.from_numpy(ph).to(d) if P else torch.zeros(1, device=d), P, lo, hi, so, b_t, cls, ev,
                        ci, si, cnt)
    torch.cuda.synchronize()
    c = cnt.cpu().numpy()
    return cls[:P].cpu().numpy(), ev[:P].cpu().numpy(), ci.cpu().numpy(), si.cpu().numpy(), c


@pytest.mark.parametrize("P,n,b_t", [(64, 4, 0), (128, 8, 0), (384, 32, 128), (384, 16, 128), (1, 4, 0), (0, 4, 0),
                                     (1024, 4, 0), (1025, 8, 100), (5000, 16, 1700), (37, 8, 1), (64, 4, 1000)])
def test_select_commit_matches_oracle(P, n, b_t):
    say("select_commit P=%d n=%d b_t=%d" % (P, n, b_t))
    rng = np.random.default_rng(P * 31 + n)
    k = rng.integers(0, n + 1, P)
    ph = (k.astype(np.float32) / np.float32(n)).astype(np.float32)
    for so in (1.0, 0.75):
        cls, ev, ci, si, cnt = _select(ph, 0.125, 0.75, so, b_t)
        wcls, wev, wci, wsi, wcnt = al.select_commit(ph, 0.125, 0.75, so, b_t)
        assert np.array_equal(cnt, wcnt)
        assert np.array_equal(cls, wcls) and np.array_equal(ev, wev)
        assert np.array_equal(ci[:cnt[0]], wci) and np.array_equal(si[:cnt[1]], wsi)
        assert (ci[cnt[0]:] == -1).all() and (si[cnt[1]:] == -1).all()     # nothing written past the counts


def test_select_commit_degenerate_batches():
    for ph in (np.zeros(70, np.float32), np.ones(70, np.float32), np.full(70, 0.5, np.float32),
               np.array([0.125, 0.75, np.nextafter(np.float32(0.125), np.float32(0)),
                         np.nextafter(np.float32(0.75), np.float32(1))], np.float32)):
        got = _select(ph, 0.125, 0.75, 1.0, 0)
        want = al.select_commit(ph, 0.125, 0.75, 1.0, 0)
        assert np.array_equal(got[4], want[4]) and np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
        assert np.array_equal(got[2][:want[4][0]], want[2])


@pytest.mark.parametrize("sizes", [[8] * 29, [16] * 91, [128] * 128, [2, 0, 5, 1, 33]])
def test_advantages_match_oracle(sizes):
    import paper_2605_26606_amd as pc
    say("advantages sizes=%s..." % sizes[:3])
    d = "cuda"
    r, off = workloads.make_binary_rewards(sizes, seed=sum(sizes))
    for eps in (1e-6, 0.0):
        adv = torch.full((max(len(r), 1),), 5.0, device=d)
        mu = torch.zeros(len(sizes), device=d)
        sg = torch.zeros(len(sizes), device=d)
        pc.pc_advantages(torch.from_numpy(r).to(d), torch.from_numpy(off).to(d), eps, adv, mu, sg)
        torch.cuda.synchronize()
        wadv, wmu, wsg = al.advantages(r, off, eps)
        assert np.array_equal(adv[:len(r)].cpu().numpy(), wadv)
        assert np.array_equal(mu.cpu().numpy(), wmu) and np.array_equal(sg.cpu().numpy(), wsg)
        # per-group invariants of Section 3.2
        a = adv[:len(r)].cpu().numpy().astype(np.float64)
        for p in range(len(sizes)):
            g = a[off[p]:off[p + 1]]
            assert abs(g.sum()) < 1e-4
            assert g[g > 0].sum() <= len(g) / 2 + 1e-5
    # float rewards
    rng = np.random.default_rng(1)
    r = rng.random(int(off[-1])).astype(np.float32)
    adv = torch.zeros(len(r), device=d)
    pc.pc_advantages(torch.from_numpy(r).to(d), torch.from_numpy(off).to(d), 1e-6, adv)
    torch.cuda.synchronize()
    wadv, _, _ = al.advantages(r, off, 1e-6)
    got = adv.cpu().numpy()
    assert np.abs(got - wadv).max() <= 2.4e-7 * max(1.0, np.abs(wadv).max())


def test_variance_filter_bit_exact():
    # pc_select_commit_var against the oracle's reading for rewards that are not binary: multi-valued rewards, all
    # three classes, caps, thresholds hit exactly; and, on 0/1 rewards with thresholds p (1 - p), the same output as
    # pc_select_commit (Section 4.2 thresholds)
    import paper_2605_26606_amd as pc
    d = "cuda"
    rng = np.random.default_rng(12)
    for P, G, levels, b_t in ((64, 4, 3, 0), (1000, 8, 5, 100), (5000, 16, 11, 0), (3, 4, 2, 1), (1, 4, 3, 0)):
        r = (rng.integers(0, levels, P * G) / float(levels - 1)).astype(np.float32)
        r.reshape(P, G)[: P // 4] = np.round(r.reshape(P, G)[: P // 4])          # some binary groups
        off = (np.arange(P + 1) * G).astype(np.int32)
        mean = torch.empty(P, device=d)
        var = torch.empty(P, device=d)
        pc.pc_group_stats(torch.from_numpy(r).to(d), torch.from_numpy(off).to(d), None, None, mean, var)
        _, _, wmean, wvar = al.group_stats(r, off)
        assert np.array_equal(mean.cpu().numpy(), wmean)
        assert np.abs(var.cpu().numpy() - wvar).max() <= 1e-7
        mean_h, var_h = mean.cpu().numpy(), var.cpu().numpy()
        for vh, ve, pv, so in ((0.109375, 0.1875, 0.5, 1.0), (0.05, 0.05, 0.4, 0.8), (0.0, 0.3, 0.5, 2.0)):
            cls = torch.full((P,), 9, dtype=torch.uint8, device=d)
            ev = torch.full((P,), 9, dtype=torch.uint8, device=d)
            ci = torch.full((P,), -1, dtype=torch.int32, device=d)
            si = torch.full((P,), -1, dtype=torch.int32, device=d)
            cnt = torch.zeros(4, dtype=torch.int32, device=d)
            pc.pc_select_commit_var(mean, var, P, vh, ve, pv, so, b_t, cls, ev, ci, si, cnt)
            torch.cuda.synchronize()
            wcls, wev, wci, wsi, wcnt = al.select_commit_variance(mean_h, var_h, vh, ve, pv, so, b_t)
            assert np.array_equal(cls.cpu().numpy(), wcls) and np.array_equal(ev.cpu().numpy(), wev)
            assert np.array_equal(cnt.cpu().numpy(), wcnt)
            assert np.array_equal(ci.cpu().numpy()[:wcnt[0]], wci) and (ci.cpu().numpy()[wcnt[0]:] == -1).all()
            assert np.array_equal(si.cpu().numpy()[:wcnt[1]], wsi) and (si.cpu().numpy()[wcnt[1]:] == -1).all()
    # binary truth table through both entry points
    for n in (4, 8, 16, 32):
        groups = np.concatenate([np.r_[np.ones(k, np.float32), np.zeros(n - k, np.float32)] for k in range(n + 1)])
        off = (np.arange(n + 2) * n).astype(np.int32)
        P = n + 1
        mean = torch.empty(P, device=d)
        var = torch.empty(P, device=d)
        pc.pc_group_stats(torch.from_numpy(groups).to(d), torch.from_numpy(off).to(d), None, None, mean, var)
        outs = []
        for which in ("binary", "variance"):
            cls = torch.empty(P, dtype=torch.uint8, device=d)
            ev = torch.empty(P, dtype=torch.uint8, device=d)
            ci = torch.full((P,), -1, dtype=torch.int32, device=d)
            si = torch.full((P,), -1, dtype=torch.int32, device=d)
            cnt = torch.zeros(4, dtype=torch.int32, device=d)
            if which == "binary":
                pc.pc_select_commit(mean, P, 0.125, 0.75, 1.0, 3, cls, ev, ci, si, cnt)
            else:
                pc.pc_select_commit_var(mean, var, P, 0.125 * 0.875, 0.75 * 0.25, 0.5, 1.0, 3, cls, ev, ci, si, cnt)
            torch.cuda.synchronize()
            outs.append([t.cpu().numpy() for t in (cls, ev, ci, si, cnt)])
        for a, b in zip(*outs):
            assert np.array_equal(a, b)
