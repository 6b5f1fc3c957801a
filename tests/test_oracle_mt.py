"""The oracle's timing variant (row copies of a call spread over host threads) gives the bytes of the plain,
single-threaded oracle: it is only ever used as a reported baseline, never as the parity reference."""
import numpy as np
import pytest

import rb_workloads as wl
from oracle import rbo


@pytest.mark.parametrize("threads", [1, 3, 8])
@pytest.mark.parametrize("K,S,row_bytes,b,c,r", [
    (5, 3, 4096, 64, 40, 20),        # few slots: several candidates of a step land on one slot, in list order
    (1, 2, 48, 16, 16, 4),           # rows shorter than one 64-byte slice per thread
    (40, 50, 1000, 128, 16, 16),     # row length not a multiple of the slice unit
])
def test_threaded_copies_give_the_plain_oracles_bytes(threads, K, S, row_bytes, b, c, r):
    rng = np.random.default_rng(7)
    plain, spread = rbo.Buffer(K, S, row_bytes), rbo.Buffer(K, S, row_bytes)
    pool = rbo.Pool(threads)
    for t in range(40):
        x = rng.integers(0, 256, (b, row_bytes), dtype=np.uint8)
        y = rng.integers(0, K, b)
        plain.update(x, y, c, 3, t)
        spread.update_mt(pool, x, y, c, 3, t)
        ref = np.full((r, row_bytes), 9, dtype=np.uint8)
        n1, x1, y1 = plain.sample_augment(r, 3, t, out_x=ref.copy())
        n2, x2, y2 = spread.sample_augment_mt(pool, r, 3, t, out_x=ref.copy())
        assert n1 == n2 and np.array_equal(y1, y2) and np.array_equal(x1, x2)
    assert np.array_equal(plain.fill, spread.fill) and np.array_equal(plain.buf_y, spread.buf_y)
    assert np.array_equal(plain.export_rows(0, K * S), spread.export_rows(0, K * S))
    pool.close()


def test_threaded_variant_on_the_tiny_workload_and_its_limits():
    w = wl.C1
    plain, spread = rbo.Buffer(w.K, w.S, w.row_bytes), rbo.Buffer(w.K, w.S, w.row_bytes)
    pool = rbo.Pool(4)
    for t in range(w.steps):
        x, y = wl.make_batch(w, t)
        hx, hy = wl.as_row_bytes(x), y.numpy()
        plain.update(hx, hy, w.c, w.lib_seed, t)
        spread.update_mt(pool, hx, hy, w.c, w.lib_seed, t)
        a, b = plain.sample_augment(w.r, w.lib_seed, t), spread.sample_augment_mt(pool, w.r, w.lib_seed, t)
        assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert np.array_equal(plain.export_rows(0, w.K * w.S), spread.export_rows(0, w.K * w.S))
    # the reduced-precision storage form converts while it copies: not served by the threaded variant
    narrow = rbo.Buffer(4, 2, 32)
    narrow.set_storage(rbo.STORE_BF16)
    with pytest.raises(ValueError):
        narrow.update_mt(pool, np.zeros((4, 32), dtype=np.uint8), np.zeros(4, dtype=np.int64), 2, 0, 0)
    with pytest.raises(ValueError):
        rbo.Pool(0)
    pool.close()
