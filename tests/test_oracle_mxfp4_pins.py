"""Pins of the oracle's MXFP4 conversion (OCP Microscaling Formats specification: E2M1 elements, E8M0
block scale over 32 values) against the format's definition, worked by hand, and against invariants."""
import numpy as np

import oracle

GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def dequant(codes, scales):
    mag = GRID[codes & 7] * np.where(codes & 8, -1.0, 1.0)
    return mag * np.repeat(2.0 ** (scales.astype(np.int32) - 127), 32, axis=1)


def test_hand_worked_block():
    """Largest magnitude 6: floor(log2 6) = 2, shared exponent 0, byte 127; representable values map to
    themselves, halfway points go to the neighbour whose mantissa bit is 0, 7 saturates to 6."""
    v = np.zeros((1, 32))
    v[0, :8] = GRID
    v[0, 8:20] = [-0.5, -6, 0.25, 0.75, 1.25, 1.75, 2.5, 5.0, 3.5, 0.26, 0.24, 7.0]
    codes, scales = oracle.mxfp4_quantize(v)
    assert scales.tolist() == [[127]]
    assert codes[0, :8].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    #                                -0.5 -6  .25 .75 1.25 1.75 2.5 5  3.5 .26 .24 7
    assert codes[0, 8:20].tolist() == [9, 15, 0, 2, 2, 4, 4, 6, 6, 1, 0, 7]
    assert not codes[0, 20:].any()


def test_block_scale_is_floor_log2_minus_two():
    for amax, byte in [(1.0, 125), (1.999, 125), (2.0, 126), (4.0, 127), (7.99, 127), (8.0, 128), (2.0 ** -20, 105),
                       (3.0 * 2.0 ** 10, 136)]:
        v = np.zeros((1, 64))
        v[0, 5] = -amax                 # block 0
        v[0, 40] = amax / 4             # block 1: its own scale, two binades lower
        _, scales = oracle.mxfp4_quantize(v)
        assert scales[0, 0] == byte and scales[0, 1] == byte - 2, (amax, scales)


def test_zero_block_and_tiny_values():
    v = np.zeros((2, 32))
    v[1, 3] = 2.0 ** -140               # below 2^-127 * 0.25 after the clamp of the exponent: rounds to zero
    codes, scales = oracle.mxfp4_quantize(v)
    assert not scales.any() and not (codes & 7).any()


def test_nearest_representable_brute_force():
    """Every code is a nearest representable value of v / 2^e (checked against all 15 values), the error is at
    most half the local step, and only values above 6 saturate."""
    rng = np.random.default_rng(11)
    v = rng.standard_normal((64, 256)) * np.exp(rng.standard_normal((64, 256)))
    codes, scales = oracle.mxfp4_quantize(v)
    e = np.repeat(scales.astype(np.int32) - 127, 32, axis=1)
    r = v.astype(np.float32).astype(np.float64) / 2.0 ** e
    assert np.abs(r).reshape(64, 8, 32).max(axis=2).min() >= 4.0 and np.abs(r).max() < 8.0
    allv = np.concatenate([-GRID[:0:-1], GRID])
    dist = np.abs(np.clip(r, -6, 6)[..., None] - allv).min(axis=-1)
    got = GRID[codes & 7] * np.where(codes & 8, -1.0, 1.0)
    assert np.array_equal(np.abs(got - np.clip(r, -6, 6)), dist)
    assert np.array_equal((codes & 7) == 7, np.abs(r) > 5.0)
    assert np.all(np.abs(dequant(codes, scales) - v.astype(np.float32))[np.abs(r) <= 6] <= 2.0 ** e[np.abs(r) <= 6])


def test_sign_and_power_of_two_equivariance():
    rng = np.random.default_rng(12)
    v = rng.standard_normal((8, 128))
    c0, s0 = oracle.mxfp4_quantize(v)
    c1, s1 = oracle.mxfp4_quantize(-v)
    assert np.array_equal(c1, c0 ^ 8) and np.array_equal(s1, s0)
    c2, s2 = oracle.mxfp4_quantize(v * 2.0 ** 9)
    assert np.array_equal(c2, c0) and np.array_equal(s2.astype(int), s0.astype(int) + 9)


def test_ties_go_to_even_code():
    """All seven halfway points, scaled into a block whose largest value fixes the exponent at 0."""
    ties = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    want = [0, 2, 2, 4, 4, 6, 6]
    v = np.zeros((1, 32))
    v[0, 0] = 4.0
    v[0, 1:8] = ties
    v[0, 8:15] = -ties
    v[0, 15:22] = np.nextafter(ties.astype(np.float32), np.float32(10)).astype(np.float64)     # just above: rounds up
    codes, _ = oracle.mxfp4_quantize(v)
    assert codes[0, 1:8].tolist() == want
    assert codes[0, 8:15].tolist() == [w | 8 for w in want]
    assert codes[0, 15:22].tolist() == [1, 2, 3, 4, 5, 6, 7]
