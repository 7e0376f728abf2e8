"""Pins for the oracle's Walsh-Hadamard transform (the yardstick of Section 4.3's speed-up figure).

The oracle evaluates the definition H_n[i][j] = (-1)^popcount(i & j) output by output; the pins tie it to
things fixed elsewhere: cases worked by hand, the library's Hadamard matrix, and the identities every
orthonormal Hadamard transform satisfies.
"""
import json
import os

import numpy as np
import pytest
import scipy.linalg

import oracle

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hadamard_small.json")


def test_hand_worked_cases():
    for case in json.load(open(GOLD))["cases"]:
        x = np.asarray([case["x"]], dtype=np.float16)
        n = x.shape[1]
        got = oracle.fwht(x)[0] * np.sqrt(n)
        assert np.allclose(got, case["expect_times_sqrt_n"], atol=1e-12), case["name"]


@pytest.mark.parametrize("n", [2, 8, 64, 1024])
def test_equals_the_library_hadamard_matrix(n):
    rs = np.random.default_rng(n)
    x = rs.standard_normal((3, n)).astype(np.float16)
    want = x.astype(np.float64) @ scipy.linalg.hadamard(n).astype(np.float64).T / np.sqrt(n)
    assert np.max(np.abs(oracle.fwht(x) - want)) <= 1e-12 * np.sqrt(n) * 8


def test_involution_and_norm():
    # H H^T = n I: the orthonormal transform is its own inverse and preserves the row norm.
    rs = np.random.default_rng(7)
    n = 256
    x = rs.standard_normal((4, n)).astype(np.float16)
    y = oracle.fwht(x)
    assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x.astype(np.float64), axis=1), rtol=1e-13)
    # second application on values that are exactly representable in fp16: +-1 rows
    s = np.where(rs.integers(0, 2, (2, n)) > 0, 1.0, -1.0).astype(np.float16)
    h = scipy.linalg.hadamard(n)[[5, 77]].astype(np.float16)          # two rows of H_n: their transform is sqrt(n) e_k
    back = oracle.fwht(h)
    want = np.zeros((2, n)); want[0, 5] = np.sqrt(n); want[1, 77] = np.sqrt(n)
    assert np.allclose(back, want, atol=1e-12)
    assert np.all(np.abs(np.abs(oracle.fwht(s) * np.sqrt(n)) % 2.0) < 1e-9)   # sums of n (even) odd numbers are even


def test_constant_and_delta_rows():
    n = 128
    ones = np.ones((1, n), dtype=np.float16)
    y = oracle.fwht(ones)[0]
    assert abs(y[0] - np.sqrt(n)) < 1e-12 and np.all(np.abs(y[1:]) < 1e-12)
    d = np.zeros((1, n), dtype=np.float16); d[0, 37] = 2.0
    y = oracle.fwht(d)[0] * np.sqrt(n)
    assert np.array_equal(y, 2.0 * scipy.linalg.hadamard(n)[:, 37])


def test_a_planted_mistake_is_seen():
    # sequency (Walsh) ordering instead of Sylvester ordering permutes the outputs: the n = 4 delta case tells them apart
    x = np.asarray([[0.0, 0.0, 1.0, 0.0]], dtype=np.float16)
    assert list(oracle.fwht(x)[0] * 2.0) == [1.0, 1.0, -1.0, -1.0]
    with pytest.raises(ValueError):
        oracle.fwht(np.zeros((1, 12), dtype=np.float16))
