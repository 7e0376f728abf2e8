"""Several linears on the same activations, each with its own transform, in one launch
(paro_rotated_linear_multi): every part against the oracle, and so is the separate call on the same part
(the two may sum in different orders, so they are not compared bit for bit)."""
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


def _parts(P, seed, T, c_in, c_outs, n_layers=8, plan=True, packed=True, bias_on=None):
    import torch
    base = pin.make_custom(seed, T, c_in, c_outs[0], n_outlier=3)
    x = base.x
    rots, ws, refs = [], [], []
    for k, c_out in enumerate(c_outs):
        li = pin.make_custom(seed + 10 * (k + 1), T, c_in, c_out, n_layers=n_layers)      # its own pairs, angles, scales, weight
        bias = pin.make_bias(seed, k, c_out) if bias_on == k else None
        rot = P.Rotation(li.pairs, li.theta, li.ch_scale)
        if plan:
            P.paro_rotation_plan_build(rot)
        w = P.W4Weight(li.qweight, li.scales, li.qzeros, bias=bias)
        if packed:
            P.paro_w4_repack(w)
        u = oracle.rotate_scale(x, li.pairs, li.theta, li.ch_scale)
        y = oracle.linear(u, li.qweight, li.scales, li.qzeros, bias)
        allowed = linear_allowed(oracle.row_sqnorms(li.qweight, li.scales, li.qzeros), u)
        rots.append(rot); ws.append(w); refs.append((y, allowed))
    return torch.as_tensor(x).cuda(), rots, ws, refs


@pytest.mark.parametrize("case", [
    dict(T=1, c_in=1024, c_outs=(16 * 13, 64, 48)),                 # q / k / v-like: three transforms, one launch
    dict(T=3, c_in=2048, c_outs=(16 * 37, 16 * 5), bias_on=1),      # gate / up-like, with a bias on one part
    dict(T=4, c_in=512, c_outs=(512, 64, 64, 16 * 9)),              # four parts, single K-slice (no exchange)
    dict(T=1, c_in=1024, c_outs=(256,)),                            # one part
    dict(T=9, c_in=1024, c_outs=(16 * 13, 64)),                     # too many tokens for one launch: sequence of calls
    dict(T=2, c_in=1024, c_outs=(128, 64), plan=False),             # no plan: sequence of calls
])
def test_multi_matches_oracle_and_separate_calls(P, case):
    import torch
    say(f"multi {case}")
    x, rots, ws, refs = _parts(P, 2000 + case["T"] + case["c_in"], case["T"], case["c_in"], case["c_outs"],
                               plan=case.get("plan", True), bias_on=case.get("bias_on"))
    need = P.paro_workspace_bytes_multi(rots, ws, case["T"])
    wsp = P.Workspace(need)
    ys = P.paro_rotated_linear_multi(rots, ws, x, wsp)
    torch.cuda.synchronize()
    for k, (y, allowed) in enumerate(refs):
        got = ys[k].cpu().numpy().astype(np.float64)
        worst = float((np.abs(got - y) / allowed).max())
        say(f"  part {k}: worst err/allowed = {worst:.3f}")
        assert worst <= 1.0
        single = P.paro_rotated_linear(rots[k], ws[k], x, P.Workspace(P.paro_workspace_bytes(rots[k], ws[k], case["T"])))
        worst_s = float((np.abs(single.cpu().numpy().astype(np.float64) - y) / allowed).max())
        assert worst_s <= 1.0, worst_s
    # a second call on the same workspace gives the same bits (exchange state left clean)
    ys2 = P.paro_rotated_linear_multi(rots, ws, x, wsp)
    assert all((a == b).all() for a, b in zip(ys, ys2))
    if case["T"] <= 4 and case.get("plan", True):
        assert wsp.partials_clean() and wsp.error_word() == 0


def test_multi_qkv_shape_of_the_8b_layer(P):
    """q 4096->4096, k and v 4096->1024 with three transforms (the layer shape the paper's models have)."""
    import torch
    say("multi qkv 8B")
    x, rots, ws, refs = _parts(P, 2100, 1, 4096, (4096, 1024, 1024))
    wsp = P.Workspace(P.paro_workspace_bytes_multi(rots, ws, 1))
    ys = P.paro_rotated_linear_multi(rots, ws, x, wsp)
    torch.cuda.synchronize()
    for k, (y, allowed) in enumerate(refs):
        assert float((np.abs(ys[k].cpu().numpy().astype(np.float64) - y) / allowed).max()) <= 1.0
