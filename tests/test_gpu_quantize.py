"""GPU parity of the quantisers (paro_w4_quantize and the activation-side ones) against Eq. 1.

The oracle evaluates Eq. 1 in fp64 on the fp64 (transformed) values; the GPU rotates and decides
in fp32.  A value that sits within the fp32 rounding of a decision boundary may legitimately fall
on either side, so the gate is the definition itself, not equality with another implementation:
the stored scale must be fp16((max - min) / 15) up to one fp16 ulp, and each zero point and code
must lie within half a step of its real-valued target min/s resp. w/s + z under the GPU's own
stored scale and zero point, plus the fp32 tolerance (quotient rounding 2^-20 relative; with a
rotation 2^-18 of the group norm, the floor the activation-side gate uses, in units of the step).
On top of that nearly all integers must equal the fp64 oracle's.
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


def _check_against_eq1(w64, codes, scales_rg, zeros_rg, rot_tol, min_agree):
    """w64 [R][C] real-valued inputs; codes [R][C]; scales_rg / zeros_rg [R][G] as stored by the GPU.
    Checks Eq. 1 from its definition and counts agreement with the fp64 oracle."""
    R, C = w64.shape
    G = C // 128
    w4 = w64.reshape(R, G, 128)
    mn, mx = w4.min(axis=2), w4.max(axis=2)
    # scale: fp16((max - min) / 15) with the 2^-14 floor, within one fp16 ulp (positive: compare bit patterns)
    s_def = np.maximum((mx - mn) / 15.0, 2.0 ** -14).astype(np.float16)
    ds = np.abs(scales_rg.view(np.uint16).astype(np.int32) - s_def.view(np.uint16).astype(np.int32))
    assert ds.max() <= 1, ds.max()
    s = scales_rg.astype(np.float64)[:, :, None]
    z = zeros_rg.astype(np.float64)[:, :, None]
    norm = np.linalg.norm(w4, axis=2, keepdims=True)
    tol = 0.5 + rot_tol * norm / s + 2.0 ** -20 * (np.abs(w4).max(axis=2, keepdims=True) / s + 16)
    zt = np.clip(-mn[:, :, None] / s, 0, 15)
    assert np.all(np.abs(z - zt) <= tol), "zero point outside its rounding interval"
    qt = np.clip(w4 / s + z, 0, 15)
    c4 = codes.reshape(R, G, 128).astype(np.float64)
    bad = np.abs(c4 - qt) > tol
    assert not bad.any(), f"{bad.sum()} codes outside their rounding interval"
    rc, rs, rz = oracle.rtn_quantize(w64)                              # scales / zeros [G][R]
    same_s = scales_rg.view(np.uint16) == rs.T.view(np.uint16)
    same = (same_s & (zeros_rg == rz.T))[:, :, None]
    agree = (c4 == rc.reshape(R, G, 128))[np.broadcast_to(same, c4.shape)]
    say(f"  scales identical {same_s.mean():.5f}, zeros identical {(zeros_rg == rz.T).mean():.5f}, codes identical {agree.mean():.6f}")
    assert same_s.mean() >= min(min_agree, 0.97) and agree.mean() >= min_agree, (same_s.mean(), agree.mean())


@pytest.mark.parametrize("shape", [(8, 128), (64, 512), (264, 1536)])
def test_plain_rtn_follows_eq1(P, shape):
    say(f"quantize plain {shape}")
    w16 = pin.make_dense_weight(300 + shape[0], *shape)
    _, _, codes, scales, zeros = _gpu_quantize(P, w16)
    _check_against_eq1(w16.astype(np.float64), codes, scales.T.copy(), zeros.T.copy(), 0.0, 0.9999)


def test_plain_rtn_degenerate_groups(P):
    say("quantize degenerate groups")
    w16 = pin.make_dense_weight(310, 16, 256)
    w16[0, :128] = 0                     # constant group: scale floor
    w16[1, :128] = np.float16(0.5)       # constant non-zero
    w16[2, 128:] = np.abs(w16[2, 128:])  # all positive: zero point clamps at 0
    w16[3, :] = -np.abs(w16[3, :])       # all negative
    _, _, codes, scales, zeros = _gpu_quantize(P, w16)
    _check_against_eq1(w16.astype(np.float64), codes, scales.T.copy(), zeros.T.copy(), 0.0, 0.9999)
    # the degenerate groups have unique answers (hand-derivable from Eq. 1 and the stated readings)
    assert float(scales[0, 0]) == 2.0 ** -14 and zeros[0, 0] == 0 and not codes[0, :128].any()   # all-zero group
    assert float(scales[0, 1]) == 2.0 ** -14 and zeros[0, 1] == 0 and (codes[1, :128] == 15).all()   # constant 0.5: saturates
    assert zeros[1, 2] == 0 and zeros[0, 3] == 15 and zeros[1, 3] == 15


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
    _check_against_eq1(wt, codes, scales.T.copy(), zeros.T.copy(), 2.0 ** -18, 0.999)


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
    no_rot = case["n_layers"] == 0
    _check_against_eq1(u, codes, scales, zeros, 0.0 if no_rot else 2.0 ** -18, 0.9999 if no_rot else 0.999)


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
        # no rotation: products of two fp16 values are exact in fp32 and in fp64, power-of-two scaling and the
        # threshold compares are exact in both, so every decision is unique
        assert np.array_equal(scales, rs)
        assert np.array_equal(got, E2M1[rc & 7] * np.where(rc & 8, -1.0, 1.0))
