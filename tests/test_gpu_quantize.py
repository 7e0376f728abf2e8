"""GPU parity of the weight-side quantiser (paro_w4_quantize) against the oracle.

Without a rotation every output is unique and must match bit for bit.  With a rotation the GPU
rotates in fp32 and the oracle in fp64, so a value that sits within the rotation's rounding of a
decision boundary may legitimately fall on either side: scales may differ by one fp16 ulp, and
each zero point and code is checked against the oracle's fp64 transformed weight with the GPU's
own scale and zero point, allowing half a step plus the rotation tolerance (2^-18 of the group
norm, the same floor the activation-side gate uses, in units of the step).
"""
import sys

import numpy as np
import pytest

import oracle
import paro_inputs as pin
from paro_tol import linear_allowed

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2511_10645_amd as paro
    assert torch.cuda.is_available()
    paro.lib()
    return paro


def _gpu_quantize(P, w16, li=None, scale=True, scale_order=0):
    import torch
    rot = None
    if li is not None:
        rot = P.Rotation(li.pairs, li.theta, li.ch_scale if scale else None, scale_order=scale_order)
        P.paro_rotation_plan_build(rot)
    W = torch.as_tensor(w16).cuda()
    q = P.paro_w4_quantize(rot, W)
    torch.cuda.synchronize()
    codes = oracle.unpack_codes(q.qweight.cpu().numpy().view(np.uint32))
    zeros = oracle.unpack_zeros(q.qzeros.cpu().numpy().view(np.uint32))
    return q, rot, codes, q.scales.cpu().numpy(), zeros


@pytest.mark.parametrize("shape", [(8, 128), (64, 512), (264, 1536)])
def test_plain_rtn_bit_exact(P, shape):
    say(f"quantize plain {shape}")
    w16 = pin.make_dense_weight(300 + shape[0], *shape)
    _, _, codes, scales, zeros = _gpu_quantize(P, w16)
    rc, rs, rz = oracle.rtn_quantize(oracle.weight_transform(w16, None, None))
    assert np.array_equal(scales.view(np.uint16), rs.view(np.uint16))
    assert np.array_equal(zeros, rz)
    assert np.array_equal(codes, rc)


def test_plain_rtn_degenerate_groups(P):
    say("quantize degenerate groups")
    w16 = pin.make_dense_weight(310, 16, 256)
    w16[0, :128] = 0                     # constant group: scale floor
    w16[1, :128] = np.float16(0.5)       # constant non-zero
    w16[2, 128:] = np.abs(w16[2, 128:])  # all positive: zero point clamps at 0
    w16[3, :] = -np.abs(w16[3, :])       # all negative
    _, _, codes, scales, zeros = _gpu_quantize(P, w16)
    rc, rs, rz = oracle.rtn_quantize(oracle.weight_transform(w16, None, None))
    assert np.array_equal(scales.view(np.uint16), rs.view(np.uint16))
    assert np.array_equal(zeros, rz) and np.array_equal(codes, rc)


@pytest.mark.parametrize("case", [
    dict(seed=401, c_in=256, c_out=8, n_layers=8, ppl=64, scale=True, order=0),
    dict(seed=402, c_in=512, c_out=72, n_layers=8, ppl=64, scale=True, order=1),
    dict(seed=403, c_in=1536, c_out=264, n_layers=8, ppl=64, scale=False, order=0),
    dict(seed=404, c_in=512, c_out=40, n_layers=3, ppl=17, scale=True, order=0),
    dict(seed=405, c_in=256, c_out=16, n_layers=0, ppl=1, scale=True, order=0),
    dict(seed=406, c_in=4096, c_out=6144, n_layers=8, ppl=64, scale=True, order=0),      # the 8B-class QKV shape
])
def test_rotated_rtn_against_oracle(P, case):
    say(f"quantize rotated {case}")
    li = pin.make_custom(case["seed"], 1, case["c_in"], case["c_out"], n_layers=case["n_layers"],
                         pairs_per_layer=case["ppl"])
    w16 = pin.make_dense_weight(case["seed"] + 50, case["c_out"], case["c_in"])
    _, _, codes, scales, zeros = _gpu_quantize(P, w16, li, case["scale"], case["order"])
    wt = oracle.weight_transform(w16, li.pairs, li.theta, li.ch_scale if case["scale"] else None,
                                 scale_order=case["order"])
    rc, rs, rz = oracle.rtn_quantize(wt)
    N, C = wt.shape
    G = C // 128
    # scales: at most one fp16 ulp apart (positive values: compare bit patterns)
    ds = np.abs(scales.view(np.uint16).astype(np.int32) - rs.view(np.uint16).astype(np.int32))
    assert ds.max() <= 1, ds.max()
    assert (ds == 0).mean() > 0.97
    # zero points and codes: valid for the GPU's own scale within half a step + rotation tolerance
    w4 = wt.reshape(N, G, 128)
    s = scales.astype(np.float64).T[:, :, None]                       # [N][G][1]
    z = zeros.astype(np.float64).T[:, :, None]
    norm = np.linalg.norm(w4, axis=2, keepdims=True)
    tol = 0.5 + 2.0 ** -18 * norm / s + 1e-6 * 16
    zt = np.clip(-w4.min(axis=2, keepdims=True) / s, 0, 15)
    assert np.all(np.abs(z - zt) <= tol), "zero point outside its rounding interval"
    qt = np.clip(w4 / s + z, 0, 15)
    c4 = codes.reshape(N, G, 128).astype(np.float64)
    bad = np.abs(c4 - qt) > tol
    assert not bad.any(), f"{bad.sum()} codes outside their rounding interval"
    # and almost always the very same integers as the oracle where scale and zero agree
    same = (ds.T == 0)[:, :, None] & (zeros == rz).T[:, :, None]
    agree = (c4 == rc.reshape(N, G, 128))[np.broadcast_to(same, c4.shape)]
    assert agree.mean() > 0.999, agree.mean()


def test_quantize_then_linear_end_to_end(P):
    """dense W -> transform + RTN on the GPU -> repack -> fused linear reproduces W.x to within the
    quantisation error, and the transform makes that error smaller on outlier-heavy weights."""
    import torch
    say("quantize end to end")
    c_in, c_out, T = 1024, 512, 3
    li = pin.make_custom(420, T, c_in, c_out, n_outlier=5)
    w16 = pin.make_dense_weight(421, c_out, c_in, outlier_frac=0.01, outlier_mult=25.0)
    y_ref = li.x.astype(np.float64) @ w16.astype(np.float64).T
    x = torch.as_tensor(li.x).cuda()

    errs = {}
    for name, use_rot in (("plain", False), ("rotated", True)):
        q, rot, codes, scales, zeros = _gpu_quantize(P, w16, li if use_rot else None, scale=False)
        P.paro_w4_repack(q)
        ws = P.Workspace(P.paro_workspace_bytes(rot, q, T))
        y = torch.empty(T, c_out, dtype=torch.float16, device="cuda")
        if use_rot:
            P.paro_rotated_linear(rot, q, x, ws, y)
        else:
            P.paro_w4a16_linear(q, x, ws, y)
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        # the linear itself is exact to its own tolerance against the oracle on the produced codes
        qw = q.qweight.cpu().numpy().view(np.uint32); qz = q.qzeros.cpu().numpy().view(np.uint32)
        u = oracle.rotate_scale(li.x, li.pairs, li.theta, None) if use_rot else li.x.astype(np.float64)
        y_q = oracle.linear(u, qw, scales, qz)
        allowed = linear_allowed(oracle.row_sqnorms(qw, scales, qz), u)
        assert np.all(np.abs(got - y_q) <= allowed + np.abs(y_q) * 2.0 ** -11)
        errs[name] = np.linalg.norm(got - y_ref) / np.linalg.norm(y_ref)
    say(f"  relative output error: {errs}")
    assert errs["rotated"] < 0.9 * errs["plain"], errs
    assert errs["rotated"] < 0.2


@pytest.mark.parametrize("case", [
    dict(seed=501, T=1, c_in=512, n_layers=8, ppl=64, order=0),
    dict(seed=502, T=7, c_in=1536, n_layers=8, ppl=64, order=1),
    dict(seed=503, T=33, c_in=256, n_layers=3, ppl=17, order=0),
    dict(seed=504, T=5, c_in=512, n_layers=0, ppl=1, order=0),
    dict(seed=505, T=16, c_in=4096, n_layers=8, ppl=64, order=0),
])
def test_activation_int4_after_rotation(P, case):
    """Transformed activations quantised per (token, group) by Eq. 1: same gate as the rotated weights."""
    import torch
    say(f"activation int4 {case}")
    li = pin.make_custom(case["seed"], case["T"], case["c_in"], 8, n_layers=case["n_layers"], pairs_per_layer=case["ppl"],
                         n_outlier=3)
    rot = P.Rotation(li.pairs, li.theta, li.ch_scale, scale_order=case["order"])
    P.paro_rotation_plan_build(rot)
    codes_t, scales_t, zeros_t = P.paro_rotate_scale_quantize_int4(rot, torch.as_tensor(li.x).cuda())
    torch.cuda.synchronize()
    codes = oracle.unpack_codes(codes_t.cpu().numpy().view(np.uint32))                  # [T][C]
    scales = scales_t.cpu().numpy()                                                      # [T][G]
    zeros = zeros_t.cpu().numpy()
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=case["order"])
    rc, rs, rz = oracle.rtn_quantize(u)                                                  # scales / zeros [G][T]
    T, C = u.shape
    G = C // 128
    ds = np.abs(scales.view(np.uint16).astype(np.int32) - rs.T.view(np.uint16).astype(np.int32))
    assert ds.max() <= 1, ds.max()
    u4 = u.reshape(T, G, 128)
    s = scales.astype(np.float64)[:, :, None]
    z = zeros.astype(np.float64)[:, :, None]
    tol = 0.5 + 2.0 ** -18 * np.linalg.norm(u4, axis=2, keepdims=True) / s + 1e-6 * 16
    assert np.all(np.abs(z - np.clip(-u4.min(axis=2, keepdims=True) / s, 0, 15)) <= tol)
    c4 = codes.reshape(T, G, 128).astype(np.float64)
    assert np.all(np.abs(c4 - np.clip(u4 / s + z, 0, 15)) <= tol)
    same = ((ds == 0) & (zeros == rz.T))[:, :, None]
    agree = (c4 == rc.reshape(T, G, 128))[np.broadcast_to(same, c4.shape)]
    assert agree.mean() > 0.999, agree.mean()
    if case["n_layers"] == 0 and case["order"] == 0:
        # no rotation: products of two fp16 values are exact in fp32, every decision is unique
        assert np.array_equal(codes, rc) and np.array_equal(zeros, rz.T)


E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


@pytest.mark.parametrize("case", [
    dict(seed=601, T=1, c_in=512, n_layers=8, ppl=64, order=0),
    dict(seed=602, T=7, c_in=1536, n_layers=8, ppl=64, order=1),
    dict(seed=603, T=33, c_in=256, n_layers=3, ppl=17, order=0),
    dict(seed=604, T=5, c_in=512, n_layers=0, ppl=1, order=0),
    dict(seed=605, T=16, c_in=4096, n_layers=8, ppl=64, order=0),
])
def test_activation_mxfp4_after_rotation(P, case):
    """Transformed activations in MXFP4: block exponent and E2M1 codes against the oracle's conversion of the
    oracle's fp64 transform; a decision may differ only where the fp32 rotation error crosses a threshold."""
    import torch
    say(f"activation mxfp4 {case}")
    li = pin.make_custom(case["seed"], case["T"], case["c_in"], 8, n_layers=case["n_layers"], pairs_per_layer=case["ppl"],
                         n_outlier=3)
    rot = P.Rotation(li.pairs, li.theta, li.ch_scale, scale_order=case["order"])
    P.paro_rotation_plan_build(rot)
    codes_t, scales_t = P.paro_rotate_scale_quantize_mxfp4(rot, torch.as_tensor(li.x).cuda())
    torch.cuda.synchronize()
    codes = oracle.unpack_codes(codes_t.cpu().numpy().view(np.uint32))                  # [T][C] nibbles
    scales = scales_t.cpu().numpy()                                                      # [T][C/32]
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=case["order"])
    rc, rs = oracle.mxfp4_quantize(u)
    T, C = u.shape
    de = scales.astype(np.int32) - rs.astype(np.int32)
    assert np.abs(de).max() <= 1 and (de != 0).mean() < 1e-3, (np.abs(de).max(), (de != 0).mean())
    # with the kernel's own exponent, every code is a nearest representable value up to the rotation's error
    e = np.repeat(scales.astype(np.int32) - 127, 32, axis=1)
    r = np.clip(u / 2.0 ** e, -6, 6)
    allv = np.concatenate([-E2M1[:0:-1], E2M1])
    best = np.abs(r[..., None] - allv).min(axis=-1)
    got = E2M1[codes & 7] * np.where(codes & 8, -1.0, 1.0)
    gnorm = np.repeat(np.linalg.norm(u.reshape(T, C // 128, 128), axis=2), 128, axis=1)
    tol = 2.0 ** -18 * gnorm / 2.0 ** e + 1e-6
    assert np.all(np.abs(got - r) <= best + tol)
    same = np.repeat(de == 0, 32, axis=1)
    mag_agree = ((codes & 7) == (rc & 7))[same]
    assert mag_agree.mean() > 0.999, mag_agree.mean()
    nz = same & ((codes & 7) != 0) & ((rc & 7) != 0)
    assert np.array_equal((codes & 8)[nz], (rc & 8)[nz])
    if case["n_layers"] == 0 and case["order"] == 0:
        # no rotation: products of two fp16 values are exact in fp32, every decision is unique
        assert np.array_equal(scales, rs)
        assert np.array_equal(got, E2M1[rc & 7] * np.where(rc & 8, -1.0, 1.0))
