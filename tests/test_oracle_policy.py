"""Pins of the oracle's buffer policy (CPU only): Algorithm 1 and the sampling
rule of Sec. IV-C, checked against closed forms, library routines, invariants,
a brute-force Python re-statement and the distributions the paper states."""
import numpy as np
import pytest
from scipy import stats

import pyref
import rb_workloads as wl
from oracle import rbo


def _rows(rng, b, row_bytes=16):
    return rng.integers(0, 256, (b, row_bytes), dtype=np.uint8)


# ---------------------------------------------------------------- update ---

def test_all_candidates_from_empty_is_a_stable_counting_sort():
    # c = b removes the random selection; with room for everything the sub-buffer
    # of class k is the mini-batch rows labelled k in mini-batch order.
    rng = np.random.default_rng(0)
    K, S, b = 7, 64, 64
    x, y = _rows(rng, b), rng.integers(0, K, b)
    buf = rbo.Buffer(K, S, 16)
    buf.update(x, y, b, seed=3, step=0)
    order = np.argsort(y, kind="stable")
    counts = np.bincount(y, minlength=K)
    assert buf.fill.tolist() == counts.tolist()
    at = 0
    for k in range(K):
        for s in range(counts[k]):
            assert np.array_equal(buf.row(k, s), x[order[at]])
            assert buf.buf_y[k, s] == k
            at += 1
        for s in range(counts[k], S):
            assert buf.row(k, s) is None and buf.buf_y[k, s] == -1


def test_single_slot_keeps_the_last_candidate_of_each_class():
    # S = 1: the slot is always 0, so class k holds the selected candidate of label k
    # with the highest mini-batch position of the latest step that had one.
    rng = np.random.default_rng(1)
    K, b, c = 5, 32, 12
    buf = rbo.Buffer(K, 1, 16)
    want = {}
    for step in range(30):
        x, y = _rows(rng, b), rng.integers(0, K, b)
        buf.update(x, y, c, seed=8, step=step)
        for pos in sorted(rbo.floyd(8, step, rbo.SELECT, b, c).tolist()):
            want[int(y[pos])] = x[pos].copy()
        for k in range(K):
            if k in want:
                assert np.array_equal(buf.row(k, 0), want[k]) and buf.fill[k] == 1
            else:
                assert buf.row(k, 0) is None and buf.fill[k] == 0


def test_single_class_appends_in_order():
    # K = 1 with room for everything (the single-class case the paper mentions for
    # generative models): the buffer is every step's candidates, in mini-batch order.
    rng = np.random.default_rng(2)
    b, c, steps = 16, 5, 20
    buf = rbo.Buffer(1, c * steps, 16)
    want = []
    for step in range(steps):
        x = _rows(rng, b)
        buf.update(x, np.zeros(b, dtype=np.int64), c, seed=1, step=step)
        want += [x[p] for p in sorted(rbo.floyd(1, step, rbo.SELECT, b, c).tolist())]
    assert buf.fill[0] == c * steps
    for s, row in enumerate(want):
        assert np.array_equal(buf.row(0, s), row)


@pytest.mark.parametrize("K,S,b,c,r", [(3, 2, 8, 5, 3), (4, 3, 12, 12, 20), (1, 4, 6, 3, 2), (10, 20, 16, 4, 4), (2, 1, 9, 9, 1)])
def test_against_bruteforce_python(K, S, b, c, r):
    rng = np.random.default_rng(K * 100 + S)
    buf, ref = rbo.Buffer(K, S, 16), pyref.PyBuffer(K, S)
    for step in range(40):
        x, y = _rows(rng, b), rng.integers(0, K, b)
        buf.update(x, y, c, seed=5, step=step)
        ref.update([bytes(v) for v in x], y.tolist(), c, seed=5, step=step)
        stored = ref.stored()
        assert buf.fill.tolist() == [len(ref.R[k]) for k in range(K)]
        for k, s, row in stored:
            assert bytes(buf.row(k, s)) == row and buf.buf_y[k, s] == k
        n, ox, oy = buf.sample_augment(r, seed=5, step=step)
        picks = ref.sample(r, seed=5, step=step)
        assert n == len(picks) == min(r, len(stored))
        for j, (k, s, row) in enumerate(picks):
            assert oy[j] == k and bytes(ox[j]) == row
        assert np.all(oy[n:] == -1)


def test_invariants_on_the_tiny_workload():
    # Workload C1 end to end: fill = min(inserted, S); a slot of class k only ever
    # holds a sample that arrived with label k; untouched slots stay untouched.
    w = wl.C1
    buf = rbo.Buffer(w.K, w.S, w.row_bytes)
    inserted = np.zeros(w.K, dtype=np.int64)
    seen = {}                                   # row bytes -> label it arrived with
    replaced = collided = 0
    for step in range(w.steps):
        x, y = wl.make_batch(w, step)
        xb, y = wl.as_row_bytes(x), y.numpy()
        for i in range(w.b):
            seen[xb[i].tobytes()] = int(y[i])
        before = buf.fill
        buf.update(xb, y, w.c, w.lib_seed, step)
        pos, cls, slot = buf.last_insertions()
        assert len(pos) == w.c and np.all(np.diff(pos) > 0)          # exactly c, ascending positions
        assert np.array_equal(cls, y[pos])
        np.add.at(inserted, cls, 1)
        assert buf.fill.tolist() == np.minimum(inserted, w.S).tolist()
        for p, k, s in zip(pos, cls, slot):
            replaced += before[k] >= w.S
        collided += len(set(zip(cls.tolist(), slot.tolist()))) < len(pos)
        fill, by = buf.fill, buf.buf_y
        for k in range(w.K):
            assert np.all(by[k, :fill[k]] == k) and np.all(by[k, fill[k]:] == -1)
            for s in range(w.S):
                row = buf.row(k, s)
                assert (row is None) == (s >= fill[k])
                if row is not None:
                    assert seen[row.tobytes()] == k
        # sampling: distinct filled slots, labels and bytes of those slots
        n, ox, oy = buf.sample_augment(w.r, w.lib_seed, step)
        F = int(fill.sum())
        g = buf.last_sampled_g()
        assert n == min(w.r, F) and len(set(g.tolist())) == n and np.all((g >= 0) & (g < F))
        k_of = np.searchsorted(np.cumsum(fill), g, side="right")   # class-major numbering, by a library routine
        s_of = g - (np.cumsum(fill) - fill)[k_of]
        for j in range(n):
            assert oy[j] == k_of[j] and np.array_equal(ox[j], buf.row(k_of[j], s_of[j]))
    assert replaced > 50          # the workload does reach the replace path
    assert buf.fill.sum() == w.K * w.S or inserted.min() < w.S


def test_bad_labels_are_skipped_and_flagged():
    rng = np.random.default_rng(4)
    K, S, b = 4, 8, 8
    x = _rows(rng, b)
    y = np.array([0, -1, 1, K, 2, 10**12, 3, -7], dtype=np.int64)
    buf = rbo.Buffer(K, S, 16)
    assert buf.flags == 0
    buf.update(x, y, b, seed=0, step=0)
    assert buf.flags & 1
    assert buf.fill.tolist() == [1, 1, 1, 1]
    for k, pos in enumerate((0, 2, 4, 6)):
        assert np.array_equal(buf.row(k, 0), x[pos])


def test_argument_validation():
    with pytest.raises(ValueError):
        rbo.Buffer(0, 1, 16)
    buf = rbo.Buffer(2, 2, 16)
    x, y = np.zeros((4, 16), dtype=np.uint8), np.zeros(4, dtype=np.int64)
    with pytest.raises(ValueError):
        buf.update(x, y, 5, 0, 0)          # c > b
    with pytest.raises(ValueError):
        buf.update(x, y, -1, 0, 0)
    buf.update(x, y, 0, 0, 0)              # c = 0 is a legal no-op
    assert buf.fill.sum() == 0


def test_replacement_is_uniform_over_the_slots():
    # A full class receiving one candidate per step: the replaced slot is uniform on [0, S),
    # whatever the age of the sample it holds (Sec. IV-B: recent and old samples are replaced alike).
    S, steps = 20, 20000
    buf = rbo.Buffer(1, S, 16)
    x = np.zeros((S, 16), dtype=np.uint8)
    buf.update(x, np.zeros(S, dtype=np.int64), S, seed=0, step=0)       # fill the class
    counts = np.zeros(S, dtype=np.int64)
    one = np.zeros((1, 16), dtype=np.uint8)
    for step in range(1, steps + 1):
        buf.update(one, np.zeros(1, dtype=np.int64), 1, seed=0, step=step)
        counts[buf.last_insertions()[2][0]] += 1
    assert stats.chisquare(counts).pvalue > 1e-4


def test_survival_of_an_original_sample():
    # After n replacements an original representative survives with probability (1 - 1/S)^n.
    S, n_rep, trials = 8, 10, 4000
    survived = 0
    for seed in range(trials):
        buf = rbo.Buffer(1, S, 16)
        x = np.arange(S, dtype=np.uint8)[:, None].repeat(16, 1) + 1
        buf.update(x, np.zeros(S, dtype=np.int64), S, seed=seed, step=0)
        new = np.zeros((1, 16), dtype=np.uint8)
        for step in range(1, n_rep + 1):
            buf.update(new, np.zeros(1, dtype=np.int64), 1, seed=seed, step=step)
        survived += buf.row(0, 3)[0] == 4
    p = (1 - 1 / S) ** n_rep
    assert abs(survived - trials * p) < 5 * np.sqrt(trials * p * (1 - p))


def test_last_writer_wins_inside_one_step():
    # Several candidates of one full class in one step may draw the same slot; the
    # one with the highest mini-batch position must be what the slot holds afterwards.
    rng = np.random.default_rng(6)
    S, b = 3, 16
    buf = rbo.Buffer(1, S, 16)
    buf.update(_rows(rng, S), np.zeros(S, dtype=np.int64), S, seed=2, step=0)
    saw_collision = False
    for step in range(1, 50):
        x = _rows(rng, b)
        buf.update(x, np.zeros(b, dtype=np.int64), b, seed=2, step=step)
        pos, _, slot = buf.last_insertions()
        assert pos.tolist() == list(range(b))
        for s in range(S):
            writers = pos[slot == s]
            saw_collision |= len(writers) > 1
            if len(writers):
                assert np.array_equal(buf.row(0, s), x[writers.max()])
    assert saw_collision


# -------------------------------------------------------------- sampling ---

def test_sampling_more_than_stored_returns_everything_once():
    rng = np.random.default_rng(9)
    K, S, b = 6, 5, 10
    buf = rbo.Buffer(K, S, 16)
    buf.update(_rows(rng, b), rng.integers(0, K, b), 7, seed=1, step=0)
    F = int(buf.fill.sum())
    sentinel = np.full((F + 3, 16), 0xAB, dtype=np.uint8)
    n, ox, oy = buf.sample_augment(F + 3, seed=1, step=0, out_x=sentinel)
    assert n == F and np.all(oy[F:] == -1) and np.all(ox[F:] == 0xAB)     # rows beyond n untouched
    got = sorted((int(k), bytes(row)) for k, row in zip(oy[:F], ox[:F]))
    want = sorted((k, bytes(buf.row(k, s))) for k in range(K) for s in range(buf.fill[k]))
    assert got == want


def test_sampling_from_empty_buffer():
    buf = rbo.Buffer(3, 3, 16)
    n, ox, oy = buf.sample_augment(4, 0, 0)
    assert n == 0 and np.all(oy == -1) and not ox.any()
    n, _, oy = buf.sample_augment(0, 0, 0)
    assert n == 0 and len(oy) == 0


def test_sampling_subsets_are_uniform_over_stored_samples():
    # F = 5 stored samples spread unevenly over classes, r = 2: 10 subsets, 1/10 each;
    # uniform over samples, so the fuller class is drawn more often (Sec. IV-C).
    buf = rbo.Buffer(3, 4, 16)
    x = (np.arange(5, dtype=np.uint8)[:, None] + np.zeros((1, 16), dtype=np.uint8))
    buf.update(x, np.array([0, 2, 2, 2, 0]), 5, seed=0, step=0)
    assert buf.fill.tolist() == [2, 0, 3]
    ids = {(a, b_): i for i, (a, b_) in enumerate((a, b_) for a in range(5) for b_ in range(a + 1, 5))}
    counts = np.zeros(10, dtype=np.int64)
    per_class = np.zeros(3, dtype=np.int64)
    for step in range(40000):
        n, ox, oy = buf.sample_augment(2, seed=4, step=step)
        a, b_ = sorted(int(v) for v in ox[:, 0])
        counts[ids[(a, b_)]] += 1
        np.add.at(per_class, oy, 1)
    assert stats.chisquare(counts).pvalue > 1e-4
    assert abs(per_class[2] / per_class.sum() - 3 / 5) < 0.01 and per_class[1] == 0


def test_inclusion_probability_of_a_stored_sample():
    # Every stored sample is equally likely to be drawn (Sec. IV-C, fair sampling): probability r/F per draw.
    w = wl.C1
    buf = rbo.Buffer(w.K, w.S, w.row_bytes)
    for step in range(w.steps):
        x, y = wl.make_batch(w, step)
        buf.update(wl.as_row_bytes(x), y.numpy(), w.c, w.lib_seed, step)
    F = int(buf.fill.sum())
    trials = 20000
    hits = np.zeros(F, dtype=np.int64)
    for step in range(trials):
        buf.sample_augment(w.r, seed=77, step=step)
        hits[buf.last_sampled_g()] += 1
    p = w.r / F
    assert np.all(np.abs(hits - trials * p) < 5.5 * np.sqrt(trials * p * (1 - p)))
