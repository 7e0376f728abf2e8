"""The entry point that allocates nothing (paro_rotated_linear_noalloc): through the C ABI, against
paro_rotated_linear on a caller-owned workspace, on two calls in a row, the second with a smaller input.
Both run the same kernels on the same data, so the outputs must be identical bit for bit."""
import ctypes
import sys

import numpy as np
import pytest

import paro_inputs as pin

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _setup(P, seed, T, c_in, c_out):
    import torch
    li = pin.make_custom(seed, T, c_in, c_out, n_outlier=3)
    rot = P.Rotation(li.pairs, li.theta, li.ch_scale)
    P.paro_rotation_plan_build(rot)
    w = P.W4Weight(li.qweight, li.scales, li.qzeros)
    P.paro_w4_repack(w)
    return li, rot, w, torch.as_tensor(li.x).cuda()


def test_noalloc_matches_workspace_call_twice():
    import torch
    import paper_2511_10645_amd as P
    assert torch.cuda.is_available()
    L = P.lib()
    st = torch.cuda.current_stream().cuda_stream
    # first call: 4 tokens, 8 K-slices exchanged; second call: 1 token, fewer slices and outputs
    for seed, T, c_in, c_out in ((8101, 4, 4096, 16 * 37), (8102, 1, 2048, 16 * 11)):
        say(f"noalloc T={T} {c_in}->{c_out}")
        li, rot, w, x = _setup(P, seed, T, c_in, c_out)
        ws = P.Workspace(P.paro_workspace_bytes(rot, w, T))
        want = P.paro_rotated_linear(rot, w, x, ws)
        got = torch.full((T, c_out), float("nan"), dtype=torch.float16, device="cuda")
        rc = L.paro_rotated_linear_noalloc(rot.ref(), w.ref(), x.data_ptr(), x.stride(0), got.data_ptr(), got.stride(0), T, st)
        assert rc == 0, rc
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        assert np.isfinite(got.cpu().numpy().astype(np.float32)).all()
        # and once more on the same inputs: the static array was left consistent
        got2 = torch.full_like(got, float("nan"))
        assert L.paro_rotated_linear_noalloc(rot.ref(), w.ref(), x.data_ptr(), x.stride(0), got2.data_ptr(), got2.stride(0), T, st) == 0
        torch.cuda.synchronize()
        assert torch.equal(got2, want)


def test_noalloc_rejects_what_it_cannot_serve():
    import torch
    import paper_2511_10645_amd as P
    L = P.lib()
    li, rot, w, x = _setup(P, 8103, 5, 1024, 64)            # 5 tokens: the rotation runs as a pass of its own (scratch part)
    y = torch.empty((5, 64), dtype=torch.float16, device="cuda")
    assert L.paro_rotated_linear_noalloc(rot.ref(), w.ref(), x.data_ptr(), x.stride(0), y.data_ptr(), y.stride(0), 5, None) == 5
    # exchange part beyond the static array: 10 K-slices x 4 tokens x 55296 outputs x 4 bytes (validated on the host, no launch)
    from paper_2511_10645_amd import binding as B
    FAKE = 0x10000
    rb = B._CRotation(5120, 128, 8, 64, FAKE, FAKE, FAKE, 0, FAKE)
    wb = B._CW4Weight(5120, 55296, 128, None, None, None, None, FAKE)
    assert L.paro_rotated_linear_noalloc(ctypes.byref(rb), ctypes.byref(wb), FAKE, 5120, FAKE, 55296, 4, None) == 6
    assert L.paro_rotated_linear_noalloc(None, ctypes.byref(wb), FAKE, 5120, FAKE, 55296, 1, None) == 1
