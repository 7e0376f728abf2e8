"""Algorithm A1 (selection of independent channel pairs): oracle pins and the host implementation.

No GPU: the selection runs on the host.  The oracle is pinned by a case worked by hand
(tests/golden/pair_selection_g4.json) and by the properties the algorithm guarantees; the
library's implementation must then return exactly the oracle's pairs.
"""
import json
import os

import numpy as np
import pytest

import oracle
import paro_inputs as pin
import paper_2511_10645_amd as paro

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "pair_selection_g4.json")))


def test_oracle_hand_worked_case():
    got = oracle.select_pairs(GOLD["order"], GOLD["group"], GOLD["n_rotations"], GOLD["pairs_per_rotation"])
    assert [[list(p) for p in r] for r in got] == GOLD["expect"]
    c2 = GOLD["second_case"]
    got = oracle.select_pairs(GOLD["order"], GOLD["group"], c2["n_rotations"], c2["pairs_per_rotation"])
    assert [[list(p) for p in r] for r in got] == c2["expect"]


@pytest.mark.parametrize("g,K,N,seed", [(128, 8, 64, 1), (128, 8, 40, 2), (16, 15, 8, 3), (8, 9, 4, 4)])
def test_oracle_properties(g, K, N, seed):
    order = pin.make_pair_order(seed, g)
    P = [(i, j) for i in range(g) for j in range(i + 1, g)]
    shuffled = [P[k] for k in order]
    rots = oracle.select_pairs(order, g, K, N)
    assert len(rots) == K
    used_before = set()
    for r, pr in enumerate(rots):
        assert len(pr) <= N
        ch = [c for p in pr for c in p]
        assert len(ch) == len(set(ch))                       # Def. 1: independent pairs
        assert all(i < j for i, j in pr)
        assert not (set(pr) & used_before)                   # no pair reused across rotations
        # greedy: a pair of the shuffled list that comes before the last selected one and was not
        # selected is blocked by an earlier selection of this rotation or by an earlier rotation
        if pr:
            pos = {p: k for k, p in enumerate(shuffled)}
            assert [pos[p] for p in pr] == sorted(pos[p] for p in pr)      # selection follows list order
            last = pos[pr[-1]] if len(pr) == N else len(shuffled)
            chosen_at = {}
            for p in pr:
                chosen_at[p[0]] = pos[p]; chosen_at[p[1]] = pos[p]
            for k in range(last):
                p = shuffled[k]
                if p in pr:
                    continue
                blocked_pair = p in used_before
                blocked_ch = any(c in chosen_at and chosen_at[c] < k for c in p)
                assert blocked_pair or blocked_ch, (r, p)
        used_before |= set(pr)
    # the complete graph always yields a perfect matching in the first rotation
    if N == g // 2:
        assert len(rots[0]) == N
    # all g-1 rotations of a 1-factorisation cannot exceed the pair supply
    assert sum(len(pr) for pr in rots) <= g * (g - 1) // 2


@pytest.mark.parametrize("g,K,N,seed", [(128, 8, 64, 11), (128, 8, 17, 12), (128, 1, 64, 13), (64, 8, 32, 14),
                                          (6, 7, 3, 15), (2, 2, 1, 16)])
def test_library_matches_oracle(g, K, N, seed):
    order = pin.make_pair_order(seed, g)
    pairs, counts = paro.paro_select_pairs_host(order, g, K, N)
    ref = oracle.select_pairs(order, g, K, N)
    for r in range(K):
        assert counts[r] == len(ref[r])
        assert [tuple(p) for p in pairs[r, :counts[r]].tolist()] == ref[r]
        assert not pairs[r, counts[r]:].any()                # empty slots are (0, 0)
    # what it returns is a valid pair table for the runtime (Def. 1 check of the library)
    assert paro.paro_validate_pairs_host(pairs[None], group=g) == 0


def test_library_hand_worked_case_and_errors():
    import ctypes
    pairs, counts = paro.paro_select_pairs_host(np.array(GOLD["order"], dtype=np.int32), 4, 3, 2)
    assert pairs.tolist() == GOLD["expect"] and counts.tolist() == [2, 2, 2]
    L = paro.lib()
    order = np.array(GOLD["order"], dtype=np.int32)
    out = np.zeros((3, 2, 2), dtype=np.int16)
    assert L.paro_select_pairs_host(None, 4, 3, 2, out.ctypes.data, None) == 1               # null
    assert L.paro_select_pairs_host(order.ctypes.data, 4, 3, 3, out.ctypes.data, None) == 2  # N > g/2
    assert L.paro_select_pairs_host(order.ctypes.data, 1, 3, 0, out.ctypes.data, None) == 2
    bad = order.copy(); bad[0] = bad[1]
    assert L.paro_select_pairs_host(bad.ctypes.data, 4, 3, 2, out.ctypes.data, None) == 4    # not a permutation


def test_selected_pairs_drive_the_rotation_oracle():
    # pairs chosen by Algorithm A1 are a legal transform: norm-preserving per group
    g, K = 128, 8
    order = pin.make_pair_order(21, g)
    pairs, _ = paro.paro_select_pairs_host(order, g, K, 64)
    rs = np.random.default_rng(3)
    theta = rs.uniform(-np.pi, np.pi, size=(1, K, 64)).astype(np.float32)
    x = rs.standard_normal((4, g)).astype(np.float16)
    u = oracle.rotate_scale(x, pairs[None], theta, None)
    assert np.allclose(np.linalg.norm(u, axis=1), np.linalg.norm(x.astype(np.float64), axis=1), rtol=1e-12)
