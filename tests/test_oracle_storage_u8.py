"""Pins of the oracle's 8-bit storage form (CPU only).

A binary32 value x is stored as the byte nearest to 255 x and handed out as byte / 255.  The byte is pinned to the
nearest integer of the EXACT product (rational arithmetic) wherever the binary32 rounding of the product cannot
matter, to its error bound everywhere, to the ties, to the special values, to monotonicity and to PyTorch's CPU
arithmetic (a library routine); the way back to the binary32 nearest to the exact quotient; the buffer-level
behaviour to a round trip through those routines and to the unchanged policy decisions.
"""
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import rbo


def _bits(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def _value(bits):
    return struct.unpack("<f", struct.pack("<I", bits & 0xFFFFFFFF))[0]


def _some_values():
    rng = np.random.default_rng(3)
    v = list(rng.random(4000, dtype=np.float32))                                # [0, 1)
    v += list((rng.random(1000, dtype=np.float32) * 1.5 - 0.25))               # some outside [0, 1]
    v += [np.float32(k / 255.0) for k in range(256)]                            # the values that come back out
    v += [np.nextafter(np.float32((k + 0.5) / 255.0), np.float32(d)) for k in range(255) for d in (0, 1)]   # next to the ties
    v += [np.float32((k + 0.5) / 255.0) for k in range(255)]
    return [float(x) for x in v]


def test_byte_is_the_nearest_integer_of_the_exact_product():
    half = Fraction(1, 2)
    for x in _some_values():
        exact = 255 * Fraction(x)                    # a binary32 value is a rational number: no rounding here
        q = rbo.f32_to_u8(_bits(x))
        if exact <= 0:
            assert q == 0
            continue
        if exact >= 255:
            assert q == 255
            continue
        # the binary32 product is within 2^-17 of the exact one (products below 256 have a last bit of at most 2^-16),
        # so away from the half-integers the byte is the nearest integer of the exact product ...
        below = exact.numerator // exact.denominator
        frac = exact - below
        if abs(frac - half) > Fraction(1, 2 ** 17):
            assert q == below + (1 if frac > half else 0), (x, q, float(exact))
        # ... and everywhere it is one of the two nearest, at most half a step (and that 2^-17) away
        assert abs(q - exact) <= half + Fraction(1, 2 ** 17), (x, q, float(exact))


def test_ties_go_to_the_even_byte_and_special_values_saturate():
    # products that are exactly k + 1/2 in binary32: 255 * x with x = (2k + 1) / 2 * 2^-8 * (256 / 255) is not
    # exact in general, so the ties are found by the library product itself
    rng = np.random.default_rng(5)
    ties = 0
    for k in range(255):
        for x in (np.float32((k + 0.5) / 255.0), np.nextafter(np.float32((k + 0.5) / 255.0), np.float32(0)), np.nextafter(np.float32((k + 0.5) / 255.0), np.float32(1))):
            p = np.float32(x) * np.float32(255.0)    # IEEE binary32 product
            if float(p) == k + 0.5:
                ties += 1
                assert rbo.f32_to_u8(_bits(float(x))) == (k if k % 2 == 0 else k + 1), (k, float(x))
    assert ties > 50
    assert rbo.f32_to_u8(_bits(0.0)) == 0 and rbo.f32_to_u8(0x80000000) == 0           # both zeros
    assert rbo.f32_to_u8(_bits(-0.3)) == 0 and rbo.f32_to_u8(_bits(-1e30)) == 0
    assert rbo.f32_to_u8(0x00000001) == 0 and rbo.f32_to_u8(0x007FFFFF) == 0           # subnormals
    assert rbo.f32_to_u8(_bits(1.0)) == 255 and rbo.f32_to_u8(_bits(1.0001)) == 255 and rbo.f32_to_u8(_bits(3e38)) == 255
    assert rbo.f32_to_u8(0x7F800000) == 255 and rbo.f32_to_u8(0xFF800000) == 0         # infinities
    for nan in (0x7FC00000, 0xFFC00000, 0x7F800001, 0xFFFFFFFF):
        assert rbo.f32_to_u8(nan) == 0
    assert rbo.f32_to_u8(_bits(0.5)) == 128                                            # 127.5 exactly: even neighbour


def test_byte_is_monotone_and_agrees_with_the_library_arithmetic():
    rng = np.random.default_rng(11)
    x = np.sort(np.concatenate([rng.random(200_000, dtype=np.float32), rng.random(20_000, dtype=np.float32) * 3 - 1]))
    got = np.array([rbo.f32_to_u8(int(b)) for b in x.view(np.uint32)], dtype=np.int64)
    assert np.all(np.diff(got) >= 0)
    want = torch.round(torch.from_numpy(x) * 255.0).clamp(0, 255).to(torch.int64).numpy()     # torch.round: halves to even
    assert np.array_equal(got, want)


def test_the_way_back_is_the_binary32_nearest_to_the_exact_quotient():
    for q in range(256):
        bits = rbo.u8_to_f32(q)
        y = _value(bits)
        exact = Fraction(q, 255)
        err = abs(Fraction(y) - exact)
        for neighbour in (np.nextafter(np.float32(y), np.float32(2)), np.nextafter(np.float32(y), np.float32(-1))):
            assert err <= abs(Fraction(float(neighbour)) - exact), q
        assert rbo.f32_to_u8(bits) == q                      # a value that was handed out is stored as the same byte again
    assert _value(rbo.u8_to_f32(0)) == 0.0 and _value(rbo.u8_to_f32(255)) == 1.0
    # error of a round trip for values in [0, 1]: at most half a step
    rng = np.random.default_rng(2)
    for x in rng.random(2000, dtype=np.float32):
        back = _value(rbo.u8_to_f32(rbo.f32_to_u8(_bits(float(x)))))
        assert abs(Fraction(back) - Fraction(float(x))) <= Fraction(1, 510) + Fraction(1, 2 ** 24)


@pytest.mark.parametrize("policy", [(0, 0), (1, 1), (0, 2)])
def test_buffer_with_8_bit_storage_holds_the_bytes_and_makes_the_same_decisions(policy):
    K, S, elems, b, c, r = 6, 4, 48, 32, 20, 9
    rng = np.random.default_rng(21)
    plain, small = rbo.Buffer(K, S, 4 * elems), rbo.Buffer(K, S, 4 * elems)
    small.set_storage(rbo.STORE_U8)
    assert small.stored_row_bytes == elems
    plain.set_policy(*policy)
    small.set_policy(*policy)
    quant = np.vectorize(lambda bits: rbo.f32_to_u8(int(bits)), otypes=[np.uint8])
    back = np.vectorize(lambda q: rbo.u8_to_f32(int(q)), otypes=[np.uint32])
    for t in range(30):
        x = (rng.random((b, elems), dtype=np.float32) * 1.2 - 0.1).astype(np.float32)
        y = rng.integers(0, K, b)
        plain.update(x, y, c, 7, t)
        small.update(x, y, c, 7, t)
        for a, bb in zip(plain.last_insertions(), small.last_insertions()):
            assert np.array_equal(a, bb)                                     # same positions, classes, slots
        n1, x1, y1 = plain.sample_augment(r, 7, t)
        n2, x2, y2 = small.sample_augment(r, 7, t)
        assert n1 == n2 and np.array_equal(y1, y2)
        # what comes out is what went in, through the two routines
        want = back(quant(x1[:n1].view(np.uint32))).astype(np.uint32)
        assert np.array_equal(x2[:n2].view(np.uint32), want)
    assert np.array_equal(plain.fill, small.fill) and np.array_equal(plain.buf_y, small.buf_y)
    stored = small.export_rows(0, K * S)
    full = plain.export_rows(0, K * S)
    filled = plain.buf_y.reshape(-1) >= 0
    assert np.array_equal(stored[filled], quant(full[filled].view(np.uint32)))
    with pytest.raises(ValueError):
        rbo.Buffer(2, 2, 6).set_storage(rbo.STORE_U8)                         # rows not made of 4-byte elements
