"""Pins of the oracle's random primitives (CPU only).

Philox4x32-10 is pinned to published known-answer vectors and to a separate
Python statement of the generator; the range reduction to exact big-integer
arithmetic and closed forms; Floyd's subset sampling to its defining
invariants, to a set-based Python version and to the exact uniform
distribution over subsets (chi-square).
"""
import itertools
import os

import numpy as np
import pytest
from scipy import stats

import pyref
from oracle import rbo


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 2
    for ctr, key, want in rows:
        assert list(rbo.philox4x32_10(ctr, key)) == want
        assert pyref.philox4x32_10(ctr, key) == want


def test_philox_matches_python_statement():
    rng = np.random.default_rng(7)
    for _ in range(2000):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64).tolist()
        key = rng.integers(0, 2**32, 2, dtype=np.uint64).tolist()
        assert list(rbo.philox4x32_10(ctr, key)) == pyref.philox4x32_10(ctr, key)


def test_philox_is_a_bijection_of_the_counter_lowbits():
    # For a fixed key Philox permutes the counter space: distinct counters give distinct outputs.
    outs = {tuple(rbo.philox4x32_10([i, 0, 0, 0], [5, 9])) for i in range(4096)}
    assert len(outs) == 4096


def test_philox_bit_frequencies():
    words = np.array([rbo.philox4x32_10([i, 3, 1, 0], [0, 0]) for i in range(8192)], dtype=np.uint32)
    bits = ((words[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(-1, 4 * 32)
    freq = bits.mean(axis=0)
    # each bit is a fair coin: 8192 trials, sd = 0.0055; 6 sd bound
    assert np.all(np.abs(freq - 0.5) < 0.034)


def test_draw64_counter_and_key_layout():
    seed, step, purpose, index = 0x1122334455667788, 0x99AABBCCDDEEFF00, 2, 77
    w = rbo.philox4x32_10([index, purpose, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
    assert rbo.draw64(seed, step, purpose, index) == int(w[0]) | (int(w[1]) << 32)
    assert rbo.draw64(seed, step, purpose, index) == pyref.draw64(seed, step, purpose, index)
    # every field matters
    base = rbo.draw64(1, 2, 3, 4)
    assert len({base, rbo.draw64(2, 2, 3, 4), rbo.draw64(1, 3, 3, 4), rbo.draw64(1, 2, 1, 4), rbo.draw64(1, 2, 3, 5),
                rbo.draw64(1 + 2**32, 2, 3, 4), rbo.draw64(1, 2 + 2**32, 3, 4)}) == 7


def test_bounded_exact_and_closed_forms():
    rng = np.random.default_rng(11)
    for i in range(500):
        seed, step = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**63))
        u = rbo.draw64(seed, step, 2, i)
        for n in (1, 2, 3, 7, 20, 130, 1000, 2**20, 2**31 - 1, 10**7, 2**40 + 1):
            got = rbo.bounded(seed, step, 2, i, n)
            assert got == (u * n) >> 64            # exact floor(u*n / 2^64)
            assert 0 <= got < n
        assert rbo.bounded(seed, step, 2, i, 1) == 0
        for k in (1, 5, 17, 32, 33, 63):            # a power of two keeps the top k bits of the draw
            assert rbo.bounded(seed, step, 2, i, 1 << k) == u >> (64 - k)


def test_bounded_is_uniform():
    n = 13
    counts = np.bincount([rbo.bounded(5, s, 2, 0, n) for s in range(26000)], minlength=n)
    assert stats.chisquare(counts).pvalue > 1e-4


@pytest.mark.parametrize("n,m", [(1, 1), (5, 0), (5, 5), (16, 4), (40, 13), (4096, 1024), (10**7, 64)])
def test_floyd_invariants(n, m):
    for step in range(20):
        x = rbo.floyd(3, step, 1, n, m)
        assert len(x) == m and len(set(x.tolist())) == m
        assert m == 0 or (x.min() >= 0 and x.max() < n)
        # element i of the emission order is either a draw below n-m+i+1 or exactly n-m+i
        assert all(int(x[i]) <= n - m + i for i in range(m))
        assert x.tolist() == pyref.floyd(3, step, 1, n, m)
    if m == n:
        assert sorted(x.tolist()) == list(range(n))


def test_floyd_subsets_are_uniform():
    # b = 4, c = 2: each of the 6 subsets must come up with probability 1/6.
    subsets = {s: i for i, s in enumerate(itertools.combinations(range(4), 2))}
    counts = np.zeros(6, dtype=np.int64)
    for seed in range(60):
        for step in range(1000):
            counts[subsets[tuple(sorted(rbo.floyd(seed, step, 1, 4, 2).tolist()))]] += 1
    assert counts.sum() == 60000
    assert stats.chisquare(counts).pvalue > 1e-4
    # F = 5, r = 2 with the sampling tag: 10 subsets, 1/10 each.
    subsets = {s: i for i, s in enumerate(itertools.combinations(range(5), 2))}
    counts = np.zeros(10, dtype=np.int64)
    for step in range(50000):
        counts[subsets[tuple(sorted(rbo.floyd(9, step, 3, 5, 2).tolist()))]] += 1
    assert stats.chisquare(counts).pvalue > 1e-4


@pytest.mark.parametrize("b,c", [(16, 4), (128, 16)])
def test_floyd_marginal_inclusion_probability(b, c):
    # Each sample of the mini-batch is inserted with probability c/b (Sec. IV-B).
    trials = 20000
    hits = np.zeros(b, dtype=np.int64)
    for step in range(trials):
        hits[rbo.floyd(0, step, 1, b, c)] += 1
    p = c / b
    sd = np.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(hits - trials * p) < 5 * sd)
