"""Pins of the stochastic-rounding function and its counter-based generator (Sec. 3.4)."""
import os

import numpy as np

from oracle import qgalore as Q
from oracle import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sr_hash_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#"):
            continue
        seed, step, idx, h = line.split()
        rows.append((int(seed), int(step), int(idx), int(h, 16)))
    return rows


def test_hash_known_answers_and_pure_python_twin():
    rows = _kat()
    assert len(rows) >= 8
    for seed, step, idx, h in rows:
        assert int(Q.sr_hash(seed, step, np.array([idx], dtype=np.uint64))[0]) == h
        # independent integer-only implementation
        assert brute.uniform(seed, step, idx) == (h >> 8) / 2 ** 24
    # vectorised over mixed high words
    idx = np.array([5, 2 ** 32 + 5, 7], dtype=np.uint64)
    got = Q.sr_uniform(42, 150000, idx)
    assert [float(g) for g in got] == [brute.uniform(42, 150000, int(i)) for i in idx]


def test_mixer_is_a_bijection_on_a_sample_and_avalanches():
    x = np.arange(1 << 16, dtype=np.uint64)
    assert np.unique(Q._mix32(x)).size == x.size
    # flipping one input bit flips about half of the output bits
    base = Q._mix32(x)
    for b in (0, 7, 19, 31):
        flipped = Q._mix32(x ^ np.uint64(1 << b))
        frac = np.mean([bin(int(v)).count("1") for v in (base ^ flipped)[:4096]]) / 32
        assert 0.45 < frac < 0.55


def test_uniform_range_chi2_and_correlation():
    n = 1 << 18
    idx = np.arange(n, dtype=np.uint64)
    u = Q.sr_uniform(0, 1, idx)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))           # 24-bit grid, exact in fp32
    counts = np.bincount((u * 256).astype(np.int64), minlength=256)
    chi2 = np.sum((counts - n / 256) ** 2 / (n / 256))
    assert chi2 < 255 + 5 * np.sqrt(2 * 255)                      # 5 sigma of chi2(255)
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    # lag-1 correlation across neighbouring elements and across successive steps
    c_idx = np.corrcoef(u[:-1], u[1:])[0, 1]
    u2 = Q.sr_uniform(0, 2, idx)
    c_step = np.corrcoef(u, u2)[0, 1]
    assert abs(c_idx) < 4 / np.sqrt(n) and abs(c_step) < 4 / np.sqrt(n)
    # different seeds decorrelate too
    u3 = Q.sr_uniform(1, 1, idx)
    assert abs(np.corrcoef(u, u3)[0, 1]) < 4 / np.sqrt(n)


def test_sr_is_unbiased_and_two_valued():
    # E[F_SR(x)] = x (Sec. 3.4): mean over 1e5 draws within 3 sigma
    n = 100000
    for k, x in enumerate([0.1, 0.5, 0.9, -0.3, 3.0, -2.75, 100.25]):
        idx = np.arange(n, dtype=np.uint64) + np.uint64(k * n)
        u = Q.sr_uniform(7, 1 + k, idx)
        r = Q.sr_round(np.full(n, x), u)
        assert set(np.unique(r)) <= {np.floor(x), np.ceil(x)}
        p = x - np.floor(x)
        sigma = np.sqrt(p * (1 - p) / n)
        assert abs(r.mean() - x) <= 3 * sigma + 1e-12
    # over steps for one element (the trajectory of a single weight)
    u = np.array([Q.sr_uniform(3, t, np.array([12345], dtype=np.uint64))[0] for t in range(1, 20001)])
    r = Q.sr_round(np.full(u.size, 0.27), u)
    assert abs(r.mean() - 0.27) <= 3 * np.sqrt(0.27 * 0.73 / u.size)


def test_sr_integers_are_fixed_points():
    u = Q.sr_uniform(0, 1, np.arange(4096, dtype=np.uint64))
    for v in (-128.0, -5.0, 0.0, 1.0, 64.0, 127.0):
        assert np.all(Q.sr_round(np.full(u.size, v), u) == v)
