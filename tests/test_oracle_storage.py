"""Pins of the oracle's reduced-precision storage variant (CPU only).

The binary32 -> bfloat16 conversion is pinned to the definition of round-to-nearest-even
evaluated in exact arithmetic, to special cases with known answers, to its error bound and
to PyTorch's CPU conversion (a library routine); the buffer-level behaviour to a round trip
through that library routine and to the unchanged policy decisions.
"""
import struct

import numpy as np
import pytest
import torch

from oracle import rbo


def _f(bits):
    return struct.unpack("<f", struct.pack("<I", bits & 0xFFFFFFFF))[0]


def _nearest_even_by_definition(bits):
    """bfloat16 pattern nearest to the binary32 `bits` (finite), distances taken in exact arithmetic
    (Python floats are binary64: every binary32 value and every difference of two neighbours is exact)."""
    x = _f(bits)
    down = bits >> 16
    up = down + 1
    lo, hi = _f(down << 16), _f(up << 16)
    if (up & 0x7FFF) > 0x7F80:            # `up` would not be a number: cannot happen for finite input
        raise AssertionError
    if (up & 0x7F80) == 0x7F80 and (up & 0x7F) == 0:
        # the neighbour away from zero is infinity: rounding treats it as the next power of two, 2^128
        hi = (2.0 ** 128) * (-1.0 if bits >> 31 else 1.0)
    d_lo, d_hi = abs(x - lo), abs(hi - x)
    if d_lo < d_hi:
        return down
    if d_hi < d_lo:
        return up
    return down if down % 2 == 0 else up


@pytest.mark.parametrize("upper", [0x0000, 0x0001, 0x007F, 0x0080, 0x3F80, 0x3F81, 0x4049, 0x7F7E, 0x7F7F,
                                   0x8000, 0x8001, 0xBF80, 0xC2F7, 0xFF7F])
def test_conversion_is_round_to_nearest_even_for_every_lower_half(upper):
    for lower in range(0, 0x10000, 1):
        bits = (upper << 16) | lower
        assert rbo.f32_to_bf16(bits) == _nearest_even_by_definition(bits), hex(bits)


def test_conversion_known_answers():
    cases = {
        0x00000000: 0x0000, 0x80000000: 0x8000,                  # zeros keep their sign
        0x3F800000: 0x3F80,                                      # 1.0 is representable
        0x3F808000: 0x3F80,                                      # tie between 0x3F80 (even) and 0x3F81: down
        0x3F818000: 0x3F82,                                      # tie between 0x3F81 and 0x3F82 (even): up
        0x3F808001: 0x3F81, 0x3F807FFF: 0x3F80,                  # just beside a tie
        0x7F7FFFFF: 0x7F80,                                      # largest binary32 rounds to infinity
        0x7F7F7FFF: 0x7F7F, 0x7F7F8000: 0x7F80,                  # around the largest finite bfloat16 (odd: the tie goes up)
        0xFF7FFFFF: 0xFF80,
        0x7F800000: 0x7F80, 0xFF800000: 0xFF80,                  # infinities
        0x00000001: 0x0000, 0x00008000: 0x0000, 0x00008001: 0x0001, 0x00018000: 0x0002,   # subnormals
        0x7FC00000: 0x7FC0, 0xFFC00001: 0xFFC0, 0x7F800001: 0x7FC0, 0xFF812345: 0xFFC1,   # NaN: sign and top payload kept, quiet
    }
    for bits, want in cases.items():
        assert rbo.f32_to_bf16(bits) == want, hex(bits)
    for h in (0x0000, 0x3F80, 0x7F7F, 0x8001, 0xFF80, 0x7FC1):
        assert rbo.bf16_to_f32(h) == h << 16
        assert rbo.f32_to_bf16(h << 16) == h                     # representable values come back unchanged


def test_conversion_matches_the_library_routine_on_random_patterns():
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 2**32, 200000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0, 0x80000000, 0x7F7FFFFF, 0x00000001, 0x007FFFFF, 0x00800000, 0x3F808000, 0x3F818000], dtype=np.uint32)
    bits = np.concatenate([bits, special])
    x = torch.from_numpy(bits.view(np.float32).copy())
    finite_or_inf = ~torch.isnan(x)
    want = x.to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([rbo.f32_to_bf16(int(v)) for v in bits], dtype=np.uint16)
    keep = finite_or_inf.numpy()
    assert np.array_equal(got[keep], want[keep])
    # NaN inputs give NaN outputs of the same sign
    nan_out = got[~keep]
    assert np.all((nan_out & 0x7F80) == 0x7F80) and np.all((nan_out & 0x007F) != 0)
    assert np.array_equal(nan_out >> 15, (bits[~keep] >> 31).astype(np.uint16))


def test_conversion_error_bound_and_monotonicity():
    rng = np.random.default_rng(4)
    x = np.sort(rng.standard_normal(50000).astype(np.float32) * np.float32(1e3))
    h = np.array([rbo.f32_to_bf16(int(v)) for v in x.view(np.uint32)], dtype=np.uint32)
    back = (h << 16).astype(np.uint32).view(np.float32)
    # 8 significand bits: half a unit in the last place is 2^-9 relative to the binade
    assert np.all(np.abs(back.astype(np.float64) - x.astype(np.float64)) <= np.abs(x.astype(np.float64)) * 2.0 ** -8)
    assert np.all(np.diff(back.astype(np.float64)) >= 0)         # rounding never reorders values


def test_buffer_with_bf16_storage_round_trips_through_the_library_routine():
    K, S, elems, b, c, r = 5, 4, 24, 16, 8, 6
    rng = np.random.default_rng(5)
    plain, small = rbo.Buffer(K, S, elems * 4), rbo.Buffer(K, S, elems * 4)
    small.set_storage(rbo.STORE_BF16)
    assert small.stored_row_bytes == elems * 2 and plain.stored_row_bytes == elems * 4
    for step in range(30):
        x = (rng.standard_normal((b, elems)) * 10).astype(np.float32)
        y = rng.integers(0, K, b)
        plain.update(x, y, c, 77, step)
        small.update(x, y, c, 77, step)
        # storage does not touch the policy: same insertions, same slots
        for a, bb in zip(plain.last_insertions(), small.last_insertions()):
            assert np.array_equal(a, bb)
        assert np.array_equal(plain.fill, small.fill) and np.array_equal(plain.buf_y, small.buf_y)
        pos, cls, slot = small.last_insertions()
        last = {}
        for p, k, s in zip(pos, cls, slot):
            last[(int(k), int(s))] = int(p)
        for (k, s), p in last.items():
            want = torch.from_numpy(x[p]).to(torch.bfloat16)
            assert np.array_equal(small.row(k, s), want.view(torch.uint8).numpy().reshape(-1))
        n1, px, py = plain.sample_augment(r, 77, step)
        n2, sx, sy = small.sample_augment(r, 77, step)
        assert n1 == n2 and np.array_equal(py, sy)
        # what comes back is what was stored, widened: the plain buffer's rows rounded through bfloat16
        want = torch.from_numpy(px[:n1].view(np.float32).copy()).to(torch.bfloat16).to(torch.float32).numpy()
        assert np.array_equal(sx[:n2].view(np.float32), want)
    assert np.array_equal(small.export_rows(0, K * S).shape, (K * S, elems * 2))


def test_storage_variant_is_fixed_once_the_buffer_is_in_use():
    buf = rbo.Buffer(3, 2, 16)
    with pytest.raises(ValueError):
        buf.set_storage(3)                                        # no such variant
    with pytest.raises(ValueError):
        rbo.Buffer(3, 2, 6).set_storage(rbo.STORE_BF16)           # rows are not made of 4-byte elements
    buf.set_storage(rbo.STORE_BF16)
    buf.set_storage(rbo.STORE_SAME)
    buf.update(np.zeros((4, 4), dtype=np.float32), np.zeros(4, dtype=np.int64), 2, 0, 0)
    with pytest.raises(ValueError):
        buf.set_storage(rbo.STORE_BF16)
