"""Tolerances of the parity tests, derived from the arithmetic (not from any implementation).

Rotation: results must lie within 2 fp16 ulp of the unrounded fp64 value.  The kernels keep
fp32 intermediates, so their absolute error scales with the group norm (every intermediate is
bounded by it): at most ~3 * 2^-24 * ||u_group|| per layer, 24 * 2^-24 = 0.75 * 2^-19 over 8
layers.  An output much smaller than the group norm has an arbitrarily small ulp, so the ulp is
taken at max(|ref|, 2^-10 * ||u_group||): the floor is 2^-19 * ||u_group||, just above the fp32
worst case and 128x below what fp16 intermediates would produce.

Linear: max |err| <= 5e-3 * ||w_row||_2 * ||u_t||_2 / sqrt(c_in), fp32 accumulation, where w_row
is the dequantised row and u_t the transformed activation row actually contracted.
"""
import numpy as np


def ulp16(v: np.ndarray) -> np.ndarray:
    """Spacing of binary16 at magnitude |v| (subnormal spacing 2^-24 below 2^-14)."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -14)))
    e = np.minimum(e, 15)
    return 2.0 ** (e - 10)


def rotation_check(got16: np.ndarray, ref64: np.ndarray, group: int = 128):
    """Returns (ok, worst ratio err/allowed, strict stats dict)."""
    got = got16.astype(np.float64)
    T, C = ref64.shape
    gn = np.linalg.norm(ref64.reshape(T, C // group, group), axis=2)          # rotations preserve it
    floor = np.repeat(gn * 2.0 ** -10, group, axis=1)
    allowed = 2.0 * ulp16(np.maximum(np.abs(ref64), floor))
    err = np.abs(got - ref64)
    ratio = err / allowed
    strict = err / ulp16(ref64)
    stats = {"max_ulp_strict": float(strict.max()), "frac_within_2ulp_strict": float((strict <= 2.0).mean()),
             "worst_ratio": float(ratio.max())}
    return bool((ratio <= 1.0).all()), stats


def linear_allowed(w_sqnorm: np.ndarray, u: np.ndarray) -> np.ndarray:
    """Allowed |err| per (t, n): 5e-3 * ||w_n|| * ||u_t|| / sqrt(C)."""
    un = np.linalg.norm(u, axis=1)
    return 5e-3 * np.sqrt(w_sqnorm)[None, :] * un[:, None] / np.sqrt(u.shape[1])
