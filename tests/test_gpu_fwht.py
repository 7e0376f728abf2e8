"""GPU parity of the Walsh-Hadamard yardstick (paro_fwht) against the oracle's definition.

Gate: as for the rotation, 2 fp16 ulp taken at max(|ref|, 2^-10 ||x_row||): the kernel's fp32 butterflies
carry an absolute error of at most about log2(n) 2^-24 ||x_row|| (every level adds one rounding of values bounded
by the row norm), while the ulp of a nearly cancelled output is arbitrarily small.
"""
import sys

import numpy as np
import pytest

import oracle
from paro_tol import ulp16

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _check(got16, ref):
    rn = np.linalg.norm(ref, axis=1, keepdims=True)
    allowed = 2.0 * ulp16(np.maximum(np.abs(ref), 2.0 ** -10 * rn))
    err = np.abs(got16.astype(np.float64) - ref)
    worst = float((err / allowed).max())
    strict = float((err <= 2.0 * ulp16(ref)).mean())
    say(f"  worst err/allowed {worst:.3f}, within 2 strict ulp {strict:.5f}")
    assert worst <= 1.0
    assert strict >= 0.999


@pytest.mark.parametrize("T,n", [(1, 8), (3, 16), (5, 64), (2, 128), (7, 1024), (3, 2048), (33, 4096), (2, 8192), (2, 16384), (1, 32768)])
def test_fwht_against_definition(T, n):
    import torch
    import paper_2511_10645_amd as P
    say(f"fwht T={T} n={n}")
    rs = np.random.default_rng(100 * T + n)
    x = rs.standard_normal((T, n)).astype(np.float16)
    x[:, rs.integers(0, n, 2)] *= 50                                   # outlier channels, as in the activations
    got = P.paro_fwht(torch.as_tensor(x).cuda())
    torch.cuda.synchronize()
    _check(got.cpu().numpy(), oracle.fwht(x))


def test_fwht_in_place_strided_and_twice():
    import torch
    import paper_2511_10645_amd as P
    say("fwht in place, padded rows, applied twice")
    T, n, ld = 6, 512, 512 + 24
    rs = np.random.default_rng(5)
    x = rs.standard_normal((T, n)).astype(np.float16)
    buf = torch.full((T, ld), 3.0, dtype=torch.float16, device="cuda")
    buf[:, :n] = torch.as_tensor(x).cuda()
    P.paro_fwht(buf[:, :n], buf[:, :n])
    torch.cuda.synchronize()
    _check(buf[:, :n].cpu().numpy(), oracle.fwht(x))
    assert (buf[:, n:] == 3.0).all()                                   # padding untouched
    # the orthonormal transform is its own inverse: twice gives x back up to two fp16 roundings
    back = P.paro_fwht(buf[:, :n]).cpu().numpy().astype(np.float64)
    assert np.max(np.abs(back - x.astype(np.float64))) <= 4 * 2.0 ** -11 * np.max(np.abs(x.astype(np.float64))) + 2.0 ** -10 * np.linalg.norm(x, axis=1).max() / np.sqrt(n) * 4
