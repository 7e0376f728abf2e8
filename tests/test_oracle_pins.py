"""Pins for the fp64 CPU oracle: every part is tied to something other than itself.

What fixes each part (all CPU, no GPU):
  fp16 converters  exhaustive against numpy's float16 casts (all 65536 encodings,
                   every tie between neighbours, random doubles)
  rotation         hand-computed closed forms (tests/golden, from Eq. 4 / Eq. 5),
                   per-layer norm preservation, inverse round trip, dense-matrix
                   formulation multiplied by numpy, 2-D textbook rotation,
                   commutation inside a layer (Def. 2), scale order (Eq. 8)
  unpack           every code in every nibble position, words built by hand
  dequant          exhaustive (q, z, scale) against numpy, index layout by brute force,
                   RTN error bound of Eq. 1
  linear           theta = 0 / scale = 1 reduces to numpy's X @ W^T, brute-force
                   loops on a tiny case, Eq. 2 identity with explicit matrices
"""
import json
import os

import numpy as np
import pytest

import oracle
import paro_inputs as pin

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- fp16 converters

def test_fp16_to_f64_exhaustive():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.fp16_to_f64(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_f64_to_fp16_exact_values_ties_and_random():
    bits = np.arange(0x7C00, dtype=np.uint16)          # all finite non-negative encodings
    vals = bits.view(np.float16).astype(np.float64)
    # exact values round to themselves
    assert np.array_equal(oracle.round_fp16(vals).view(np.uint16), bits)
    # midpoints between neighbours: ties go to the even mantissa; plus one ulp64 either side
    mid = 0.5 * (vals[:-1] + vals[1:])
    for probe in (mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf)):
        for sgn in (1.0, -1.0):
            with np.errstate(over="ignore"):
                want = (sgn * probe).astype(np.float16)
            got = oracle.round_fp16(sgn * probe)
            assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # overflow boundary: 65520 is the tie between 65504 and 2^16 -> inf
    edge = np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, -65520.0, 2.0 ** -25, 2.0 ** -24 * 0.5000001,
                     2.0 ** -24 * 1.5, 0.0, -0.0])
    with np.errstate(over="ignore"):
        want = edge.astype(np.float16)
    assert np.array_equal(oracle.round_fp16(edge).view(np.uint16), want.view(np.uint16))
    rng = np.random.default_rng(7)
    r = np.concatenate([rng.normal(0, 1, 200000), rng.normal(0, 300, 200000), rng.uniform(-7e-5, 7e-5, 200000)])
    assert np.array_equal(oracle.round_fp16(r).view(np.uint16), r.astype(np.float16).view(np.uint16))


# ----------------------------------------------------------------------------- rotation

def _run_case(case):
    g = case["group"]
    x = np.array([case["x"]], dtype=np.float16)
    pairs = np.array(case["pairs"], dtype=np.int16)[None]         # one group
    theta = np.array(case["theta"], dtype=np.float32)[None]
    return oracle.rotate_scale(x, pairs, theta, None, group=g)[0]


def test_rotation_closed_forms_from_golden():
    with open(os.path.join(GOLDEN, "rotation_closed_forms.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 6
    for case in cases:
        got = _run_case(case)
        # theta is stored as fp32, so cos(pi/2) is ~4e-8, not 0
        np.testing.assert_allclose(got, np.array(case["expect"]), atol=5e-7, err_msg=case["name"])


def _dense_layer(pairs_l, theta_l, g):
    """One independent rotation as an explicit g x g matrix: identity plus the
    four entries G_ii = G_jj = cos, G_ij = -sin, G_ji = +sin per pair (Eq. 4)."""
    R = np.eye(g)
    for (i, j), th in zip(pairs_l, theta_l):
        if i == j:
            continue
        c, s = np.cos(np.float64(th)), np.sin(np.float64(th))
        R[i, i] = c; R[i, j] = -s
        R[j, i] = s; R[j, j] = c
    return R


def _dense_transform(pairs_g, theta_g, g):
    R = np.eye(g)
    for l in range(pairs_g.shape[0]):
        R = _dense_layer(pairs_g[l], theta_g[l], g) @ R          # layer 1 acts first
    return R


@pytest.fixture(scope="module")
def tiny():
    return pin.make_linear(0, 0)


def test_rotation_matches_dense_matrix_product(tiny):
    u = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    x = tiny.x.astype(np.float64) * tiny.ch_scale.astype(np.float64)
    for g in range(tiny.n_groups):
        R = _dense_transform(tiny.pairs[g], tiny.theta[g], 128)
        np.testing.assert_allclose(R @ R.T, np.eye(128), atol=1e-13)
        want = x[:, g * 128:(g + 1) * 128] @ R.T
        np.testing.assert_allclose(u[:, g * 128:(g + 1) * 128], want, rtol=0, atol=1e-12 * np.abs(want).max())


def test_rotation_two_dim_textbook():
    rng = np.random.default_rng(3)
    for _ in range(20):
        th = np.float32(rng.uniform(-np.pi, np.pi))
        x = rng.normal(size=2).astype(np.float16)
        got = oracle.rotate_scale(x[None], np.array([[[[0, 1]]]], np.int16), np.array([[[th]]], np.float32), None, group=2)[0]
        c, s = np.cos(np.float64(th)), np.sin(np.float64(th))
        want = np.array([[c, -s], [s, c]]) @ x.astype(np.float64)     # counter-clockwise rotation of (u_i, u_j)
        np.testing.assert_allclose(got, want, atol=1e-15)


def test_each_layer_preserves_group_norm(tiny):
    x = tiny.x.astype(np.float64) * tiny.ch_scale.astype(np.float64)
    ref = np.linalg.norm(x.reshape(-1, 128), axis=1)
    prev = None
    for k in range(1, 9):
        u = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale, n_layers=k)
        nk = np.linalg.norm(u.reshape(-1, 128), axis=1)
        np.testing.assert_allclose(nk, ref, rtol=1e-13)
        assert prev is None or not np.array_equal(prev, u)     # every layer does something
        prev = u


def test_inverse_round_trip(tiny):
    u = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    inv_pairs = np.ascontiguousarray(tiny.pairs[:, ::-1])
    inv_theta = np.ascontiguousarray(-tiny.theta[:, ::-1])
    back = oracle.rotate_inplace(u, inv_pairs, inv_theta) / tiny.ch_scale.astype(np.float64)
    np.testing.assert_allclose(back, tiny.x.astype(np.float64), atol=1e-12 * 200)


def test_pairs_inside_a_layer_commute_bitwise(tiny):
    rng = np.random.default_rng(11)
    u0 = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    pairs = tiny.pairs.copy(); theta = tiny.theta.copy()
    for g in range(pairs.shape[0]):
        for l in range(pairs.shape[1]):
            perm = rng.permutation(64)
            pairs[g, l] = pairs[g, l][perm]; theta[g, l] = theta[g, l][perm]
    assert np.array_equal(u0, oracle.rotate_scale(tiny.x, pairs, theta, tiny.ch_scale))


def test_reversed_pair_equals_negated_angle(tiny):
    u0 = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    u1 = oracle.rotate_scale(tiny.x, np.ascontiguousarray(tiny.pairs[..., ::-1]), -tiny.theta, tiny.ch_scale)
    np.testing.assert_allclose(u1, u0, atol=1e-12)


def test_layers_do_not_commute_and_order_is_array_order(tiny):
    u0 = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    u1 = oracle.rotate_scale(tiny.x, np.ascontiguousarray(tiny.pairs[:, ::-1]),
                             np.ascontiguousarray(tiny.theta[:, ::-1]), tiny.ch_scale)
    assert np.abs(u0 - u1).max() > 1e-2


def test_scale_order_and_null_scale(tiny):
    s = tiny.ch_scale.astype(np.float64)
    plain = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, None)
    after = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale, scale_order=1)
    np.testing.assert_allclose(after, plain * s, rtol=1e-15)
    ones = np.ones_like(tiny.ch_scale)
    assert np.array_equal(plain, oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, ones))
    before = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale, scale_order=0)
    assert np.abs(before - after).max() > 1e-2          # S and R do not commute


def test_partial_matching_and_sentinels_pass_through():
    li = pin.make_custom(5, 3, 256, 8, pairs_per_layer=40)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, None)
    x = li.x.astype(np.float64)
    for g in range(2):
        touched = np.zeros(128, bool)
        for l in range(8):
            for i, j in li.pairs[g, l]:
                if i != j:
                    touched[i] = touched[j] = True
        sl = slice(g * 128, (g + 1) * 128)
        assert np.array_equal(u[:, sl][:, ~touched], x[:, sl][:, ~touched])
        R = _dense_transform(li.pairs[g], li.theta[g], 128)
        np.testing.assert_allclose(u[:, sl], x[:, sl] @ R.T, atol=1e-12)
    assert (li.pairs[:, 1::2, -1, 0] == li.pairs[:, 1::2, -1, 1]).all()      # the sentinels are really there


def test_rotate_rejects_out_of_range_index():
    x = np.zeros((1, 128), np.float16)
    pairs = np.zeros((1, 1, 1, 2), np.int16); pairs[0, 0, 0] = (0, 128)
    with pytest.raises(ValueError):
        oracle.rotate_scale(x, pairs, np.zeros((1, 1, 1), np.float32))


# ----------------------------------------------------------------------------- unpack / dequant

def test_unpack_every_code_in_every_nibble():
    for k in range(8):
        for code in range(16):
            background = 0xFFFFFFFF if code == 0 else 0
            word = (background & ~(0xF << (4 * k)) | (code << (4 * k))) & 0xFFFFFFFF
            q = np.array([[word]], dtype=np.uint32)
            got = oracle.unpack_codes(q)[0]
            assert got[k] == code
            assert all(got[m] == (15 if code == 0 else 0) for m in range(8) if m != k)


def test_unpack_inverts_generator_packing():
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 16, size=(24, 256), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_codes(pin.pack_nibbles_u32(codes)), codes)
    zeros = rng.integers(0, 16, size=(2, 24), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_zeros(pin.pack_nibbles_u32(zeros)), zeros)
    # little-endian nibble order along the row: channel 8w+k sits in bits 4k..4k+3 of word w
    q = np.zeros((1, 2), np.uint32); q[0, 1] = 0x00000A00
    got = oracle.unpack_codes(q)[0]
    assert got[10] == 0xA and got.sum() == 0xA


def test_dequant_exhaustive_q_z_scale():
    sbits = np.arange(0x7C00, dtype=np.uint16)                              # all finite non-negative fp16
    sbits = np.concatenate([sbits, sbits | 0x8000]).astype(np.uint16)       # and negative: 63488 scales
    N = sbits.size
    assert N == 63488 and N % 8 == 0
    codes = np.tile(np.repeat(np.arange(16, dtype=np.uint8), 8), (N, 1))    # [N][128], every q
    qw = pin.pack_nibbles_u32(codes)
    s64 = sbits.view(np.float16).astype(np.float64)
    for z in range(16):
        qz = pin.pack_nibbles_u32(np.full((1, N), z, np.uint8))
        W = oracle.dequant(qw, sbits.reshape(1, N), qz)
        want = (codes.astype(np.float64) - z) * s64[:, None]
        assert np.array_equal(W, want)
        with np.errstate(over="ignore"):
            assert np.array_equal(oracle.round_fp16(W).view(np.uint16), want.astype(np.float16).view(np.uint16))


def test_dequant_index_layout_brute_force():
    rng = np.random.default_rng(5)
    N, C, g = 16, 384, 128
    codes = rng.integers(0, 16, size=(N, C), dtype=np.uint8)
    zeros = rng.integers(0, 16, size=(C // g, N), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-8, 0, size=(C // g, N)) * rng.integers(1, 8, size=(C // g, N))).astype(np.float16)
    W = oracle.dequant(pin.pack_nibbles_u32(codes), scales, pin.pack_nibbles_u32(zeros))
    for n in range(N):
        for c in range(C):
            assert W[n, c] == (int(codes[n, c]) - int(zeros[c // g, n])) * float(scales[c // g, n])
    np.testing.assert_allclose(oracle.row_sqnorms(pin.pack_nibbles_u32(codes), scales, pin.pack_nibbles_u32(zeros)),
                               (W * W).sum(1), rtol=1e-14)


def test_dequant_inverts_rtn_within_half_step():
    """Quantise with Eq. 1 (here, in the test), dequantise with the oracle: |w^ - w| <= s/2."""
    rng = np.random.default_rng(9)
    N, C, g, b = 8, 256, 128, 4
    W = rng.normal(size=(N, C))
    Wg = W.reshape(N, C // g, g)
    s = ((Wg.max(-1) - Wg.min(-1)) / (2 ** b - 1)).astype(np.float16).astype(np.float64)     # stored as fp16
    z = -np.rint(Wg.min(-1) / s)
    q = np.clip(np.rint(Wg / s[..., None]) + z[..., None], 0, 2 ** b - 1)
    inside = (np.rint(Wg / s[..., None]) + z[..., None] >= 0) & (np.rint(Wg / s[..., None]) + z[..., None] <= 15)
    assert ((z >= 0) & (z <= 15)).all()
    What = oracle.dequant(pin.pack_nibbles_u32(q.reshape(N, C).astype(np.uint8)), s.T.astype(np.float16),
                          pin.pack_nibbles_u32(z.T.astype(np.uint8))).reshape(N, C // g, g)
    err = np.abs(What - Wg)
    assert (err[inside] <= 0.5 * np.broadcast_to(s[..., None], err.shape)[inside] * (1 + 1e-12)).all()
    assert inside.mean() > 0.95


# ----------------------------------------------------------------------------- linear

def test_identity_transform_reduces_to_plain_dequant_gemm(tiny):
    zero_theta = np.zeros_like(tiny.theta)
    u = oracle.rotate_scale(tiny.x, tiny.pairs, zero_theta, None)
    assert np.array_equal(u, tiny.x.astype(np.float64))
    u1 = oracle.rotate_scale(tiny.x, tiny.pairs, zero_theta, np.ones_like(tiny.ch_scale))
    assert np.array_equal(u1, u)
    W = oracle.dequant(tiny.qweight, tiny.scales, tiny.qzeros)
    y = oracle.linear(u, tiny.qweight, tiny.scales, tiny.qzeros)
    want = tiny.x.astype(np.float64) @ W.T
    np.testing.assert_allclose(y, want, atol=1e-11 * np.abs(want).max())


def test_linear_brute_force_tiny_with_bias():
    li = pin.make_custom(21, 3, 256, 16)
    bias = np.linspace(-1, 1, 16).astype(np.float16)
    u = np.random.default_rng(1).normal(size=(3, 256))
    y = oracle.linear(u, li.qweight, li.scales, li.qzeros, bias)
    for t in range(3):
        for n in range(16):
            acc = 0.0
            for c in range(256):
                acc += (int(li.codes[n, c]) - int(li.zeros[c // 128, n])) * float(li.scales[c // 128, n]) * u[t, c]
            assert abs(y[t, n] - (acc + float(bias[n]))) <= 1e-12 * max(1.0, abs(acc))
    ts = np.array([0, 2, 1, 2]); ns = np.array([15, 0, 7, 7])
    ys, ww = oracle.linear_samples(u, li.qweight, li.scales, li.qzeros, ts, ns, bias)
    assert np.array_equal(ys, y[ts, ns])
    np.testing.assert_allclose(ww, oracle.row_sqnorms(li.qweight, li.scales, li.qzeros)[ns], rtol=1e-15)


def test_equivalent_transform_identity_eq2():
    """W x = (W S^-1 R^-1)(R S x) with W unquantised, R and S explicit matrices (Eq. 2, Eq. 8)."""
    li = pin.make_custom(33, 3, 256, 8)
    rng = np.random.default_rng(4)
    W = rng.normal(size=(8, 256))
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)          # R S x from the oracle
    x = li.x.astype(np.float64)
    Wt = np.empty_like(W)
    s = li.ch_scale.astype(np.float64)
    for g in range(2):
        sl = slice(g * 128, (g + 1) * 128)
        R = _dense_transform(li.pairs[g], li.theta[g], 128)
        Wt[:, sl] = W[:, sl] @ np.diag(1.0 / s[sl]) @ np.linalg.inv(R)
    want = x @ W.T
    np.testing.assert_allclose(u @ Wt.T, want, atol=1e-10 * np.abs(want).max())


def test_planted_mistakes_are_caught(tiny):
    """A dropped layer, a wrong sign or a transposed scale table must move the result far
    beyond any tolerance used in the parity tests (checks the pins have teeth)."""
    u = oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale)
    assert np.abs(oracle.rotate_scale(tiny.x, tiny.pairs, -tiny.theta, tiny.ch_scale) - u).max() > 1.0
    assert np.abs(oracle.rotate_scale(tiny.x, tiny.pairs, tiny.theta, tiny.ch_scale, n_layers=7) - u).max() > 1.0
    y = oracle.linear(u, tiny.qweight, tiny.scales, tiny.qzeros)
    y_bad = oracle.linear(u, tiny.qweight, np.ascontiguousarray(tiny.scales[::-1]), tiny.qzeros)
    assert np.abs(y - y_bad).max() > 0.1
