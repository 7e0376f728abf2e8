"""Pins of the oracle's MXFP4 value map and of the 4-bit x 4-bit contraction Y' = Q(X T^-1) Q(T W) + b (App. A.3):
the format's value tables, a case worked by hand, and operands that the quantiser represents without loss, for which
the contraction must equal numpy's matrix product of the ORIGINAL values."""
import json
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mxfp4_linear_small.json")


def _gold():
    with open(GOLD) as f:
        return json.load(f)


def test_value_tables_of_the_format():
    g = _gold()
    codes = np.zeros((16, 32), dtype=np.uint8)
    codes[:, 0] = np.arange(16)
    v = oracle.mxfp4_dequant(codes, np.full((16, 1), 127, dtype=np.uint8))
    want = np.array(g["e2m1_values_by_code"])
    assert np.array_equal(v[:, 0], want)
    assert np.signbit(v[8, 0]) and v[8, 0] == 0.0                      # code 8 is -0
    assert not v[:, 1:].any()
    for byte, val in g["e8m0_values"].items():
        one = np.zeros((1, 32), dtype=np.uint8)
        one[0, 5] = 2                                                   # the element 1.0
        assert oracle.mxfp4_dequant(one, np.array([[int(byte)]], dtype=np.uint8))[0, 5] == val


def test_hand_worked_contraction():
    c = _gold()["case"]
    xc = np.zeros((1, 64), dtype=np.uint8)
    for k, v in c["x_codes"].items():
        xc[0, int(k)] = v
    wc = np.zeros((2, 64), dtype=np.uint8)
    for n, row in enumerate(c["w_codes"]):
        for k, v in row.items():
            wc[n, int(k)] = v
    xs = np.array([c["x_scales"]], dtype=np.uint8)
    ws = np.array(c["w_scales"], dtype=np.uint8)
    y = oracle.mxfp4_linear(xc, xs, wc, ws, np.array(c["bias"], dtype=np.float16))
    assert np.array_equal(y, np.array(c["y"]))
    # without the bias
    y0 = oracle.mxfp4_linear(xc, xs, wc, ws)
    assert np.array_equal(y0, np.array(c["y"]) - np.array(c["bias"]))


def _representable(rng, rows, C):
    """fp64 rows whose every 32-block is k * 2^e with k on the E2M1 grid and one |k| >= 4: the conversion keeps them."""
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    k = grid[rng.integers(0, 8, size=(rows, C))] * rng.choice([-1.0, 1.0], size=(rows, C))
    k = k.reshape(rows, C // 32, 32)
    k[:, :, 0] = rng.choice([4.0, 6.0, -4.0, -6.0], size=(rows, C // 32))
    e = rng.integers(-9, 10, size=(rows, C // 32, 1))
    return (k * np.exp2(e)).reshape(rows, C)


def test_lossless_operands_give_numpys_matrix_product():
    rng = np.random.default_rng(20251)
    T, N, C = 3, 5, 256
    x, w = _representable(rng, T, C), _representable(rng, N, C)
    xc, xs = oracle.mxfp4_quantize(x)
    wc, ws = oracle.mxfp4_quantize(w)
    assert np.array_equal(oracle.mxfp4_dequant(xc, xs), x)
    assert np.array_equal(oracle.mxfp4_dequant(wc, ws), w)
    bias = rng.standard_normal(N).astype(np.float16)
    y = oracle.mxfp4_linear(xc, xs, wc, ws, bias)
    assert y.shape == (T, N)
    assert np.array_equal(y, x @ w.T + bias.astype(np.float64))         # all sums exact in fp64 at these sizes


def test_contraction_is_linear_in_each_operand_and_picks_single_products():
    rng = np.random.default_rng(20252)
    C = 64
    wc = rng.integers(0, 16, size=(4, C)).astype(np.uint8)
    ws = rng.integers(120, 135, size=(4, C // 32)).astype(np.uint8)
    wv = oracle.mxfp4_dequant(wc, ws)
    for c in (0, 31, 32, 63):
        xc = np.zeros((1, C), dtype=np.uint8)
        xc[0, c] = 2                                                    # the element 1.0 at channel c
        y = oracle.mxfp4_linear(xc, np.full((1, 2), 127, dtype=np.uint8), wc, ws)
        assert np.array_equal(y[0], wv[:, c])
        y2 = oracle.mxfp4_linear(xc, np.full((1, 2), 130, dtype=np.uint8), wc, ws)
        assert np.array_equal(y2[0], 8.0 * wv[:, c])
