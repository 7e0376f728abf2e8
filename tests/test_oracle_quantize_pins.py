"""Pins for the weight-side part of the oracle (transform of Eq. 8, RTN quantiser of Eq. 1).

None of these needs a GPU.  They tie the two functions to things fixed outside them: groups
whose codes can be written down by hand from Eq. 1, the half-step error bound that Eq. 1
implies, and the equivalence of Eq. 2 with the (separately pinned) activation-side rotation.
"""
import numpy as np
import pytest

import oracle
import paro_inputs as pin


def _group(vals):
    return np.asarray(vals, dtype=np.float64).reshape(1, 128)


def test_rtn_hand_computed_groups():
    # Eq. 1 by hand.  w = k/8, k = 0..15 (each 8 times): min 0, max 15/8, s = 1/8, z = 0, q = k
    k = np.arange(128) % 16
    codes, s, z = oracle.rtn_quantize(_group(k / 8.0))
    assert float(s[0, 0]) == 0.125 and z[0, 0] == 0 and np.array_equal(codes[0], k)
    # shifted by -1: min -1, s = 1/8, z = -round(-1 / (1/8)) = 8, q = round(w/s) + 8 = k
    codes, s, z = oracle.rtn_quantize(_group(k / 8.0 - 1.0))
    assert float(s[0, 0]) == 0.125 and z[0, 0] == 8 and np.array_equal(codes[0], k)
    # all negative range [-15/8, 0]: z = 15
    codes, s, z = oracle.rtn_quantize(_group(-(k / 8.0)))
    assert float(s[0, 0]) == 0.125 and z[0, 0] == 15 and np.array_equal(codes[0], 15 - k)
    # ties go to even: w/s = 0.5 -> 0, 1.5 -> 2, 2.5 -> 2 (range 0..15 keeps s = 1)
    w = np.zeros(128); w[1] = 15.0; w[2] = 0.5; w[3] = 1.5; w[4] = 2.5
    codes, s, z = oracle.rtn_quantize(_group(w))
    assert float(s[0, 0]) == 1.0 and z[0, 0] == 0 and list(codes[0, :5]) == [0, 15, 0, 2, 2]


def test_rtn_decisions_are_taken_on_the_real_values():
    # Eq. 1 is stated over the reals: a value a hair above a half step rounds up, a hair below
    # rounds down.  A quantiser that first rounds its input or the quotient to fp32 sees 2.5
    # exactly in both cases and answers 2 twice (ties to even).
    w = np.zeros(128); w[1] = 15.0; w[2] = 2.5 + 2.0 ** -30; w[3] = 2.5 - 2.0 ** -30; w[4] = 3.5 - 2.0 ** -30
    codes, s, z = oracle.rtn_quantize(_group(w))
    assert float(s[0, 0]) == 1.0 and z[0, 0] == 0 and list(codes[0, :5]) == [0, 15, 3, 2, 3]
    # the scale is rounded to fp16 once, from the exact (max - min) / 15: range 15 * (1 + 2^-11 + 2^-30)
    # lies just above the midpoint of the fp16 neighbours 1 and 1 + 2^-10, so it rounds up;
    # an fp32 intermediate would land on the midpoint and round to the even neighbour 1.0
    w = np.zeros(128); w[1] = 15.0 * (1.0 + 2.0 ** -11 + 2.0 ** -30)
    _, s, _ = oracle.rtn_quantize(_group(w))
    assert float(s[0, 0]) == 1.0 + 2.0 ** -10


def test_rtn_constant_group_uses_scale_floor():
    codes, s, z = oracle.rtn_quantize(_group(np.zeros(128)))
    assert float(s[0, 0]) == 2.0 ** -14 and z[0, 0] == 0 and not codes.any()


def test_rtn_layout_of_outputs():
    # two rows, two groups, distinct ranges: scales / zeros are [G][N], codes [N][C]
    w = np.zeros((2, 256))
    w[0, :128] = np.linspace(0, 15, 128); w[0, 128:] = np.linspace(-30, 0, 128)
    w[1, :128] = np.linspace(-7.5, 0, 128); w[1, 128:] = np.linspace(0, 60, 128)
    codes, s, z = oracle.rtn_quantize(w)
    assert s.shape == (2, 2) and z.shape == (2, 2) and codes.shape == (2, 256)
    assert [float(v) for v in s.reshape(-1)] == [1.0, 0.5, 2.0, 4.0]       # (g0,n0) (g0,n1) (g1,n0) (g1,n1)
    assert list(z.reshape(-1)) == [0, 15, 15, 0]


def test_rtn_error_is_at_most_half_a_step():
    rs = np.random.default_rng(5)
    w = rs.standard_normal((64, 512)) * 0.03
    codes, s, z = oracle.rtn_quantize(w)
    sf = np.repeat(s.astype(np.float64).T, 128, axis=1)                    # [N][C]
    zf = np.repeat(z.astype(np.float64).T, 128, axis=1)
    deq = (codes - zf) * sf
    err = np.abs(deq - w)
    inner = (codes > 0) & (codes < 15)
    assert inner.mean() > 0.8
    assert np.all(err[inner] <= 0.5 * sf[inner] * (1 + 1e-12))
    # clamped ends: the fp16 rounding of s may push max/s + z slightly beyond 15.5
    assert np.all(err <= 1.01 * sf)
    # every group uses both ends of the code range (min -> 0, max -> 15)
    c4 = codes.reshape(64, 4, 128)
    assert np.all(c4.min(axis=2) == 0) and np.all(c4.max(axis=2) == 15)


@pytest.mark.parametrize("scale_order", [0, 1])
def test_weight_transform_preserves_the_layer_output(scale_order):
    # Eq. 2: (T W) applied to (X T^-1) gives X W.  The activation side is pinned on its own
    # (closed forms, dense-matrix product); this ties the weight side to it.
    li = pin.make_custom(91, 5, 256, 8)
    w16 = pin.make_dense_weight(7, 8, 256)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=scale_order)
    wt = oracle.weight_transform(w16, li.pairs, li.theta, li.ch_scale, scale_order=scale_order)
    y = li.x.astype(np.float64) @ w16.astype(np.float64).T
    yt = u @ wt.T
    assert np.max(np.abs(y - yt)) <= 1e-10 * np.max(np.abs(y))
    # a transposed or sign-flipped transform does not: rotate the weights with -theta instead
    bad = oracle.weight_transform(w16, li.pairs, -li.theta, li.ch_scale, scale_order=scale_order)
    assert np.max(np.abs(y - u @ bad.T)) > 1e-3 * np.max(np.abs(y))


def test_weight_transform_without_rotation_is_the_plain_weight():
    w16 = pin.make_dense_weight(8, 4, 128)
    assert np.array_equal(oracle.weight_transform(w16, None, None), w16.astype(np.float64))
    cs = np.full(128, 2.0, dtype=np.float16)
    assert np.array_equal(oracle.weight_transform(w16, None, None, cs), w16.astype(np.float64) / 2.0)


def test_rotation_spreads_isolated_outliers_before_rtn():
    # The method's premise (Section 3): isolated outliers inflate the group's range, a rotation
    # spreads them over the group, the RTN step shrinks.  Random angles are enough to see it.
    li = pin.make_custom(92, 1, 512, 8)
    w16 = pin.make_dense_weight(9, 96, 512, outlier_frac=0.01, outlier_mult=25.0)
    ones = np.ones(512, dtype=np.float16)
    plain = w16.astype(np.float64)
    wt = oracle.weight_transform(w16, li.pairs, li.theta, ones)
    def rtn_rel_err(w):
        codes, s, z = oracle.rtn_quantize(w)
        deq = (codes - np.repeat(z.astype(np.float64).T, 128, axis=1)) * np.repeat(s.astype(np.float64).T, 128, axis=1)
        return np.linalg.norm(deq - w) / np.linalg.norm(w)
    e_plain, e_rot = rtn_rel_err(plain), rtn_rel_err(wt)
    assert e_rot < 0.9 * e_plain, (e_plain, e_rot)      # seeded: 0.154 against 0.190
