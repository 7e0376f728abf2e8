"""ctypes front end of the fp64 CPU oracle (``paro_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Importers allowed: ``tests/``, the smoke check and
the CPU-baseline leg of the benchmark.  The GPU package never imports this.

Arrays are numpy, host memory.  fp16 tensors travel as their uint16 bit
patterns (``arr.view(np.uint16)``), so no float conversion happens outside the
C file's own hand-written converters.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "paro_oracle.c")
_LIB = os.path.join(_HERE, "libparo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over tokens / output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_fp16_to_f64.restype = ctypes.c_double
        L.oracle_fp16_to_f64.argtypes = [ctypes.c_uint16]
        L.oracle_f64_to_fp16.restype = ctypes.c_uint16
        L.oracle_f64_to_fp16.argtypes = [ctypes.c_double]
        L.oracle_rotate_scale.restype = ctypes.c_int
        L.oracle_rotate_inplace.restype = ctypes.c_int
        _lib = L
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def _bits(a):
    """fp16 array -> contiguous uint16 view (bit patterns)."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def threads() -> int:
    """Threads the OpenMP loops will use (all cores this process may run on)."""
    env = os.environ.get("OMP_NUM_THREADS")
    n = len(os.sched_getaffinity(0))
    return min(n, int(env)) if env and env.isdigit() else n


def fp16_to_f64(bits: np.ndarray) -> np.ndarray:
    b = _bits(bits)
    out = np.empty(b.shape, dtype=np.float64)
    lib().oracle_widen_fp16(_p(b, ctypes.c_uint16), ctypes.c_int64(b.size), _p(out, ctypes.c_double))
    return out


def round_fp16(v: np.ndarray) -> np.ndarray:
    """fp64 -> fp16 round-to-nearest-even (the oracle's own converter); returns float16."""
    v = _c(v, np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    lib().oracle_round_fp16(_p(v, ctypes.c_double), ctypes.c_int64(v.size), _p(out, ctypes.c_uint16))
    return out.view(np.float16)


def rotate_scale(x16, pairs, theta, ch_scale16=None, group=128, scale_order=0, n_layers=None) -> np.ndarray:
    """u = R_K ... R_1 . S . x per token and group, fp64 [T][C]  (Eq. 4, 5, 8).

    ``n_layers`` < K applies only the first layers (used by the per-layer pins).
    """
    xb = _bits(x16)
    T, C = xb.shape
    pairs = _c(pairs, np.int16)
    theta = _c(theta, np.float32)
    G, K, P, two = pairs.shape
    assert two == 2 and G * group == C and theta.shape == (G, K, P)
    if n_layers is not None and n_layers != K:
        pairs = np.ascontiguousarray(pairs[:, :n_layers])
        theta = np.ascontiguousarray(theta[:, :n_layers])
        K = n_layers
    sb = _bits(ch_scale16)
    u = np.empty((T, C), dtype=np.float64)
    rc = lib().oracle_rotate_scale(_p(xb, ctypes.c_uint16), ctypes.c_int64(C), ctypes.c_int32(T), ctypes.c_int32(C),
                                   ctypes.c_int32(group), ctypes.c_int32(K), ctypes.c_int32(P),
                                   _p(pairs, ctypes.c_int16), _p(theta, ctypes.c_float),
                                   _p(sb, ctypes.c_uint16), ctypes.c_int32(scale_order),
                                   _p(u, ctypes.c_double), ctypes.c_int64(C))
    if rc != 0:
        raise ValueError("pair index out of range")
    return u


def rotate_inplace(u, pairs, theta, group=128) -> np.ndarray:
    """Apply the rotation layers alone to fp64 rows (returns a new array)."""
    u = np.array(u, dtype=np.float64, order="C", copy=True)
    T, C = u.shape
    pairs = _c(pairs, np.int16)
    theta = _c(theta, np.float32)
    G, K, P, two = pairs.shape
    assert two == 2 and G * group == C and theta.shape == (G, K, P)
    rc = lib().oracle_rotate_inplace(_p(u, ctypes.c_double), ctypes.c_int64(C), ctypes.c_int32(T), ctypes.c_int32(C),
                                     ctypes.c_int32(group), ctypes.c_int32(K), ctypes.c_int32(P),
                                     _p(pairs, ctypes.c_int16), _p(theta, ctypes.c_float))
    if rc != 0:
        raise ValueError("pair index out of range")
    return u


def weight_transform(w16, pairs, theta, ch_scale16=None, group=128, scale_order=0) -> np.ndarray:
    """wt = R_K ... R_1 . diag(1/ch_scale) . w per output row and group, fp64 [N][C]  (Eq. 8, weight side).

    ``pairs`` / ``theta`` None: no rotation (scaling only, or the identity).
    """
    wb = _bits(w16)
    N, C = wb.shape
    if pairs is None:
        pairs = np.zeros((C // group, 0, 1, 2), dtype=np.int16)
        theta = np.zeros((C // group, 0, 1), dtype=np.float32)
    pairs = _c(pairs, np.int16)
    theta = _c(theta, np.float32)
    G, K, P, two = pairs.shape
    assert two == 2 and G * group == C and theta.shape == (G, K, P)
    sb = _bits(ch_scale16)
    wt = np.empty((N, C), dtype=np.float64)
    L = lib()
    L.oracle_weight_transform.restype = ctypes.c_int
    rc = L.oracle_weight_transform(_p(wb, ctypes.c_uint16), ctypes.c_int64(C), ctypes.c_int32(N), ctypes.c_int32(C),
                                   ctypes.c_int32(group), ctypes.c_int32(K), ctypes.c_int32(P),
                                   _p(pairs, ctypes.c_int16), _p(theta, ctypes.c_float),
                                   _p(sb, ctypes.c_uint16), ctypes.c_int32(scale_order),
                                   _p(wt, ctypes.c_double), ctypes.c_int64(C))
    if rc != 0:
        raise ValueError("pair index out of range")
    return wt


def rtn_quantize(wt: np.ndarray, group=128):
    """Eq. 1 per (row, group): returns codes uint8 [N][C], scales fp16 [G][N], zeros uint8 [G][N]."""
    wt = _c(wt, np.float64)
    N, C = wt.shape
    G = C // group
    codes = np.empty((N, C), dtype=np.uint8)
    scales = np.empty((G, N), dtype=np.uint16)
    zeros = np.empty((G, N), dtype=np.uint8)
    L = lib()
    L.oracle_rtn_quantize.restype = None
    L.oracle_rtn_quantize(_p(wt, ctypes.c_double), ctypes.c_int64(C), ctypes.c_int32(N), ctypes.c_int32(C),
                          ctypes.c_int32(group), _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16),
                          _p(zeros, ctypes.c_uint8))
    return codes, scales.view(np.float16), zeros


def mxfp4_quantize(u: np.ndarray):
    """OCP MXFP4 conversion of fp64 rows (rounded to fp32 first): codes uint8 [T][C] (E2M1, bit 3 = sign),
    scales uint8 [T][C/32] (E8M0: shared exponent + 127)."""
    u = _c(u, np.float64)
    T, C = u.shape
    assert C % 32 == 0
    codes = np.empty((T, C), dtype=np.uint8)
    scales = np.empty((T, C // 32), dtype=np.uint8)
    L = lib()
    L.oracle_mxfp4_quantize.restype = None
    L.oracle_mxfp4_quantize(_p(u, ctypes.c_double), ctypes.c_int64(C), ctypes.c_int32(T), ctypes.c_int32(C),
                            _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8))
    return codes, scales


def mxfp4_dequant(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """Values of MXFP4 elements: codes uint8 [T][C], scales uint8 [T][C/32] -> fp64 [T][C]."""
    codes, scales = _c(codes, np.uint8), _c(scales, np.uint8)
    T, C = codes.shape
    assert scales.shape == (T, C // 32)
    out = np.empty((T, C), dtype=np.float64)
    L = lib()
    L.oracle_mxfp4_dequant.restype = None
    L.oracle_mxfp4_dequant(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8), ctypes.c_int32(T), ctypes.c_int32(C),
                           _p(out, ctypes.c_double))
    return out


def mxfp4_linear(x_codes, x_scales, w_codes, w_scales, bias16=None) -> np.ndarray:
    """Y' = Q(X T^-1) . Q(T W) + b on MXFP4 operands (App. A.3): fp64 [T][N]."""
    xc, xs, wc, ws = _c(x_codes, np.uint8), _c(x_scales, np.uint8), _c(w_codes, np.uint8), _c(w_scales, np.uint8)
    T, C = xc.shape
    N = wc.shape[0]
    assert wc.shape == (N, C) and xs.shape == (T, C // 32) and ws.shape == (N, C // 32)
    y = np.empty((T, N), dtype=np.float64)
    bb = _bits(bias16) if bias16 is not None else None
    L = lib()
    L.oracle_mxfp4_linear.restype = None
    L.oracle_mxfp4_linear(_p(xc, ctypes.c_uint8), _p(xs, ctypes.c_uint8), ctypes.c_int32(T), _p(wc, ctypes.c_uint8),
                          _p(ws, ctypes.c_uint8), ctypes.c_int32(N), ctypes.c_int32(C),
                          _p(bb, ctypes.c_uint16) if bb is not None else None, _p(y, ctypes.c_double))
    return y


def fwht(x16) -> np.ndarray:
    """y = H_n x / sqrt(n) per row, Sylvester order (H_n[i][j] = (-1)^popcount(i & j)), fp64 [T][n]."""
    xb = _bits(x16)
    T, n = xb.shape
    y = np.empty((T, n), dtype=np.float64)
    L = lib()
    L.oracle_fwht.restype = ctypes.c_int
    rc = L.oracle_fwht(_p(xb, ctypes.c_uint16), ctypes.c_int64(n), ctypes.c_int32(T), ctypes.c_int32(n),
                       _p(y, ctypes.c_double), ctypes.c_int64(n))
    if rc != 0:
        raise ValueError("row length is not a power of two")
    return y


def unpack_codes(qweight: np.ndarray) -> np.ndarray:
    q = _c(qweight, np.uint32)
    N, C8 = q.shape
    out = np.empty((N, C8 * 8), dtype=np.uint8)
    lib().oracle_unpack_codes(_p(q, ctypes.c_uint32), ctypes.c_int32(N), ctypes.c_int32(C8 * 8), _p(out, ctypes.c_uint8))
    return out


def unpack_zeros(qzeros: np.ndarray) -> np.ndarray:
    q = _c(qzeros, np.uint32)
    G, N8 = q.shape
    out = np.empty((G, N8 * 8), dtype=np.uint8)
    lib().oracle_unpack_zeros(_p(q, ctypes.c_uint32), ctypes.c_int32(G), ctypes.c_int32(N8 * 8), _p(out, ctypes.c_uint8))
    return out


def _wargs(qweight, scales16, qzeros, group):
    q = _c(qweight, np.uint32)
    s = _bits(scales16)
    z = _c(qzeros, np.uint32)
    N, C8 = q.shape
    C = C8 * 8
    assert s.shape == (C // group, N) and z.shape == (C // group, N // 8)
    return q, s, z, N, C


def dequant(qweight, scales16, qzeros, group=128) -> np.ndarray:
    """W^[n][c] = (q - z) * s in fp64 (Eq. 1 inverted, per-group s and z)."""
    q, s, z, N, C = _wargs(qweight, scales16, qzeros, group)
    W = np.empty((N, C), dtype=np.float64)
    lib().oracle_dequant(_p(q, ctypes.c_uint32), _p(s, ctypes.c_uint16), _p(z, ctypes.c_uint32),
                         ctypes.c_int32(N), ctypes.c_int32(C), ctypes.c_int32(group), _p(W, ctypes.c_double))
    return W


def row_sqnorms(qweight, scales16, qzeros, group=128) -> np.ndarray:
    q, s, z, N, C = _wargs(qweight, scales16, qzeros, group)
    out = np.empty(N, dtype=np.float64)
    lib().oracle_row_sqnorms(_p(q, ctypes.c_uint32), _p(s, ctypes.c_uint16), _p(z, ctypes.c_uint32),
                             ctypes.c_int32(N), ctypes.c_int32(C), ctypes.c_int32(group), _p(out, ctypes.c_double))
    return out


def linear(u, qweight, scales16, qzeros, bias16=None, group=128) -> np.ndarray:
    """y[t][n] = sum_c W^[n][c] u[t][c] (+ b[n]) in fp64 (Eq. 2)."""
    u = _c(u, np.float64)
    q, s, z, N, C = _wargs(qweight, scales16, qzeros, group)
    T = u.shape[0]
    assert u.shape == (T, C)
    b = _bits(bias16)
    y = np.empty((T, N), dtype=np.float64)
    lib().oracle_linear(_p(u, ctypes.c_double), ctypes.c_int64(C), ctypes.c_int32(T),
                        _p(q, ctypes.c_uint32), _p(s, ctypes.c_uint16), _p(z, ctypes.c_uint32), _p(b, ctypes.c_uint16),
                        ctypes.c_int32(N), ctypes.c_int32(C), ctypes.c_int32(group),
                        _p(y, ctypes.c_double), ctypes.c_int64(N))
    return y


def linear_samples(u, qweight, scales16, qzeros, t_idx, n_idx, bias16=None, group=128):
    """(y[s], ||w_row(n_s)||^2) for sampled (t_s, n_s), each computed on its own."""
    u = _c(u, np.float64)
    q, s, z, N, C = _wargs(qweight, scales16, qzeros, group)
    t_idx = _c(np.asarray(t_idx, dtype=np.int32), np.int32)
    n_idx = _c(np.asarray(n_idx, dtype=np.int32), np.int32)
    assert t_idx.shape == n_idx.shape and u.shape[1] == C
    b = _bits(bias16)
    y = np.empty(t_idx.shape, dtype=np.float64)
    ww = np.empty(t_idx.shape, dtype=np.float64)
    lib().oracle_linear_samples(_p(u, ctypes.c_double), ctypes.c_int64(C),
                                _p(q, ctypes.c_uint32), _p(s, ctypes.c_uint16), _p(z, ctypes.c_uint32),
                                _p(b, ctypes.c_uint16), ctypes.c_int32(N), ctypes.c_int32(C), ctypes.c_int32(group),
                                _p(t_idx, ctypes.c_int32), _p(n_idx, ctypes.c_int32), ctypes.c_int64(t_idx.size),
                                _p(y, ctypes.c_double), _p(ww, ctypes.c_double))
    return y, ww


def select_pairs(order, group: int, n_rotations: int, pairs_per_rotation: int):
    """Selection of independent channel pairs, Algorithm A1 (Section 4.1.2), step by step.

    ``order``: the algorithm's shuffle, given as a permutation of the pair numbers of
    P = {(i, j) | 0 <= i < j < g} in lexicographic order.  A is the g x g availability matrix
    shared by all rotations (a pair is blocked once selected); A_rot is its copy for one
    rotation, in which the rows and columns of both channels of a selected pair are blocked.
    Returns (list of K lists of (i, j) in selection order).  Pure Python: small inputs only.
    """
    g = group
    P = [(i, j) for i in range(g) for j in range(i + 1, g)]
    P_shuffled = [P[int(k)] for k in order]
    A = np.ones((g, g), dtype=np.uint8)
    np.fill_diagonal(A, 0)
    out = []
    for _r in range(n_rotations):
        A_rot = A.copy()
        P_r = []
        for (i, j) in P_shuffled:
            if len(P_r) == pairs_per_rotation:
                break
            if A_rot[i, j] == 0:
                continue
            P_r.append((i, j))
            A_rot[i, :] = 0; A_rot[:, i] = 0
            A_rot[j, :] = 0; A_rot[:, j] = 0
            A[i, j] = 0; A[j, i] = 0
        out.append(P_r)
    return out
