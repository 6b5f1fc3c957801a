"""Pins of the oracle's policy variants (CPU only): Bernoulli(c/b) candidate selection
(Sec. IV-B) and replacement strategies other than the random one, which Sec. IV-A allows:
first-in-first-out and per-class reservoir sampling."""
import numpy as np
import pytest
from scipy import stats

import pyref
from oracle import rbo


def _rows(rng, b, row_bytes=16):
    return rng.integers(0, 256, (b, row_bytes), dtype=np.uint8)


def _buffer(K, S, selection=rbo.SELECT_EXACT, eviction=rbo.EVICT_UNIFORM, row_bytes=16):
    buf = rbo.Buffer(K, S, row_bytes)
    buf.set_policy(selection, eviction)
    return buf


def test_policy_can_only_be_set_on_an_empty_buffer():
    buf = rbo.Buffer(2, 2, 16)
    with pytest.raises(ValueError):
        buf.set_policy(2, 0)
    with pytest.raises(ValueError):
        buf.set_policy(0, 3)
    buf.update(np.zeros((2, 16), dtype=np.uint8), np.zeros(2, dtype=np.int64), 2, 0, 0)
    with pytest.raises(ValueError):
        buf.set_policy(0, 1)


# ---------------------------------------------------------------- Bernoulli ---

def test_bernoulli_selection_is_an_independent_coin_per_sample():
    b, c, trials = 16, 4, 20000
    buf = _buffer(1, 10**6, selection=rbo.SELECT_BERNOULLI)
    x, y = np.zeros((b, 16), dtype=np.uint8), np.zeros(b, dtype=np.int64)
    hits = np.zeros(b, dtype=np.int64)
    pair = 0
    sizes = []
    for step in range(trials):
        buf.update(x, y, c, seed=3, step=step)
        pos = buf.last_insertions()[0]
        assert np.all(np.diff(pos) > 0)                     # visited in ascending mini-batch position
        hits[pos] += 1
        pair += (0 in pos) and (1 in pos)
        sizes.append(len(pos))
        # the coin is the documented one: a uniform integer below b, heads iff below c
        want = [q for q in range(b) if rbo.bounded(3, step, rbo.COIN, q, b) < c]
        assert pos.tolist() == want
    p = c / b
    sd = np.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(hits - trials * p) < 5 * sd)       # every sample has a c/b probability to be pushed
    assert abs(pair - trials * p * p) < 5 * np.sqrt(trials * p * p)    # two samples: independent
    # number of candidates per mini-batch: Binomial(b, c/b)
    counts = np.bincount(sizes, minlength=b + 1)
    expected = stats.binom.pmf(np.arange(b + 1), b, p) * trials
    keep = expected > 5
    chi = ((counts[keep] - expected[keep]) ** 2 / expected[keep]).sum()
    assert stats.chi2.sf(chi, keep.sum() - 1) > 1e-4


def test_bernoulli_with_c_equal_b_takes_everything():
    rng = np.random.default_rng(0)
    K, S, b = 5, 40, 30
    buf = _buffer(K, S, selection=rbo.SELECT_BERNOULLI)
    x, y = _rows(rng, b), rng.integers(0, K, b)
    buf.update(x, y, b, seed=1, step=0)
    order = np.argsort(y, kind="stable")
    counts = np.bincount(y, minlength=K)
    at = 0
    for k in range(K):
        for s in range(counts[k]):
            assert np.array_equal(buf.row(k, s), x[order[at]])
            at += 1


# --------------------------------------------------------------------- FIFO ---

def test_fifo_keeps_the_most_recent_samples_of_each_class():
    # c = b removes the random selection: class k must hold its last S arrivals, arrival n in slot n mod S.
    rng = np.random.default_rng(1)
    K, S, b = 3, 5, 8
    buf = _buffer(K, S, eviction=rbo.EVICT_FIFO)
    arrivals = {k: [] for k in range(K)}
    for step in range(25):
        x, y = _rows(rng, b), rng.integers(0, K, b)
        buf.update(x, y, b, seed=9, step=step)
        for i in range(b):
            arrivals[int(y[i])].append(x[i])
        for k in range(K):
            n = len(arrivals[k])
            assert buf.fill[k] == min(n, S)
            for m in range(max(0, n - S), n):
                assert np.array_equal(buf.row(k, m % S), arrivals[k][m])


def test_fifo_more_candidates_than_slots_in_one_step():
    rng = np.random.default_rng(2)
    S, b = 3, 16
    buf = _buffer(1, S, eviction=rbo.EVICT_FIFO)
    x = _rows(rng, b)
    buf.update(x, np.zeros(b, dtype=np.int64), b, seed=0, step=0)
    for m in range(b - S, b):
        assert np.array_equal(buf.row(0, m % S), x[m])


# ---------------------------------------------------------------- reservoir ---

def test_reservoir_holds_a_uniform_sample_of_everything_offered():
    # After N offers to one class every offered sample is stored with probability S/N.
    S, N, trials = 4, 20, 6000
    kept = np.zeros(N, dtype=np.int64)
    for seed in range(trials):
        buf = _buffer(1, S, eviction=rbo.EVICT_RESERVOIR)
        for n in range(N):
            x = np.full((1, 16), n, dtype=np.uint8)
            buf.update(x, np.zeros(1, dtype=np.int64), 1, seed=seed, step=n)
        assert buf.fill[0] == S
        held = sorted(int(buf.row(0, s)[0]) for s in range(S))
        assert len(set(held)) == S
        kept[held] += 1
    p = S / N
    assert np.all(np.abs(kept - trials * p) < 5 * np.sqrt(trials * p * (1 - p)))


def test_reservoir_acceptance_probability_decays_as_s_over_n():
    S, trials = 5, 4000
    for n_before in (5, 20, 100):
        stored = 0
        for seed in range(trials):
            buf = _buffer(1, S, eviction=rbo.EVICT_RESERVOIR)
            x = np.zeros((n_before, 16), dtype=np.uint8)
            buf.update(x, np.zeros(n_before, dtype=np.int64), n_before, seed=seed, step=0)
            buf.update(np.ones((1, 16), dtype=np.uint8), np.zeros(1, dtype=np.int64), 1, seed=seed, step=1)
            stored += len(buf.last_insertions()[0])
        p = S / (n_before + 1)
        assert abs(stored - trials * p) < 5 * np.sqrt(trials * p * (1 - p))


# ------------------------------------------- all variants against brute force ---

@pytest.mark.parametrize("selection,eviction", [
    ("exact", "fifo"), ("exact", "reservoir"), ("bernoulli", "uniform"), ("bernoulli", "fifo"), ("bernoulli", "reservoir"),
])
@pytest.mark.parametrize("K,S,b,c,r", [(3, 2, 8, 5, 3), (1, 3, 10, 10, 2), (4, 6, 12, 4, 5)])
def test_variants_against_bruteforce_python(selection, eviction, K, S, b, c, r):
    sel = {"exact": rbo.SELECT_EXACT, "bernoulli": rbo.SELECT_BERNOULLI}[selection]
    ev = {"uniform": rbo.EVICT_UNIFORM, "fifo": rbo.EVICT_FIFO, "reservoir": rbo.EVICT_RESERVOIR}[eviction]
    rng = np.random.default_rng(K * 10 + S)
    buf, ref = _buffer(K, S, sel, ev), pyref.PyBuffer(K, S, selection, eviction)
    for step in range(40):
        x, y = _rows(rng, b), rng.integers(0, K, b)
        buf.update(x, y, c, seed=6, step=step)
        ref.update([bytes(v) for v in x], y.tolist(), c, seed=6, step=step)
        assert buf.fill.tolist() == [len(ref.R[k]) for k in range(K)]
        for k, s, row in ref.stored():
            assert bytes(buf.row(k, s)) == row
        n, ox, oy = buf.sample_augment(r, seed=6, step=step)
        picks = ref.sample(r, seed=6, step=step)
        assert n == len(picks)
        for j, (k, s, row) in enumerate(picks):
            assert oy[j] == k and bytes(ox[j]) == row
