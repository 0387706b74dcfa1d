"""Pins for oracle.philox: published known-answer vectors, uniformity, and
the properties the sampler's stream relies on."""
import os

import numpy as np

from oracle import philox


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], tuple(w[6:10])))
    return rows


def test_known_answer_vectors(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert philox.philox4x32_10(ctr, key) == want


def test_round_count_and_constants_matter(golden_dir):
    # the KAT distinguishes 10 rounds from 7 (another published variant): a
    # generator truncated to 7 rounds must NOT reproduce it
    ctr, key, want = _kat(golden_dir)[2]
    c = list(ctr)
    k = list(key)
    for _ in range(7):
        p0, p1 = philox.M0 * c[0], philox.M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & philox.MASK, p1 & philox.MASK,
             ((p0 >> 32) ^ c[3] ^ k[1]) & philox.MASK, p0 & philox.MASK]
        k = [(k[0] + philox.W0) & philox.MASK, (k[1] + philox.W1) & philox.MASK]
    assert tuple(c) != want


def test_uniform_is_exact_fp32_and_open_interval():
    assert philox.uniform_from_bits(0) == 0.5 / 2 ** 23
    assert philox.uniform_from_bits(0xFFFFFFFF) == 1.0 - 0.5 / 2 ** 23
    for x in (0, 1, 255, 256, 0x12345678, 0xFFFFFFFF):
        u = philox.uniform_from_bits(x)
        assert 0.0 < u < 1.0
        assert float(np.float32(u)) == u


def test_uniformity_chi_square():
    n, bins = 200_000, 64
    u = np.array([philox.sampling_uniform(1234, 77, t) for t in range(n)])
    hist, _ = np.histogram(u, bins=bins, range=(0, 1))
    chi2 = float(((hist - n / bins) ** 2 / (n / bins)).sum())
    # chi-square with 63 dof: mean 63, sd ~11.2; 130 is ~6 sd out
    assert chi2 < 130.0
    assert abs(u.mean() - 0.5) < 0.005
    # lag-1 correlation of a counter-based stream is ~0
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.01


def test_stream_depends_on_every_input():
    base = philox.sampling_uniform(3, philox.seq_uid(5, 2), 9)
    assert base == philox.sampling_uniform(3, philox.seq_uid(5, 2), 9)
    others = {
        philox.sampling_uniform(4, philox.seq_uid(5, 2), 9),
        philox.sampling_uniform(3 + (1 << 32), philox.seq_uid(5, 2), 9),   # seed high word
        philox.sampling_uniform(3, philox.seq_uid(6, 2), 9),
        philox.sampling_uniform(3, philox.seq_uid(5, 3), 9),
        philox.sampling_uniform(3, philox.seq_uid(5, 2) + (1 << 32), 9),   # uid high word
        philox.sampling_uniform(3, philox.seq_uid(5, 2), 10),
        philox.sampling_uniform(3, philox.seq_uid(5, 2), 9, domain=1),
    }
    assert base not in others and len(others) == 7


def test_seq_uid_layout():
    assert philox.seq_uid(0, 0) == 0
    assert philox.seq_uid(1, 0) == 65536
    assert philox.seq_uid(3, 7) == 3 * 65536 + 7
