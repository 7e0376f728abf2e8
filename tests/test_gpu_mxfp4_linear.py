"""GPU parity of the weight-activation linear with MXFP4 operands, Y' = Q(X T^-1) Q(T W) + b (App. A.3), through the
C ABI against the oracle's fp64 contraction of the same codes.

Tolerance.  Every product of two MXFP4 values is exact in fp32; the kernel adds them in fp32 (inside the matrix
instruction over 128 channels, then over the K-steps of a wave, then over the waves of a block) and rounds once to fp16.
With mass = sum_c |x^ w^| the accumulated rounding is at most (C/128 + 16) * 2^-23 * mass (one rounding of at most
mass * 2^-24 per addition, doubled), the final rounding half an fp16 ulp of the result, 2^-11 |y|, plus half the
smallest fp16 subnormal.  Integer work (repacking, the quantiser without a rotation) is compared bit for bit.
"""
import sys

import numpy as np
import pytest

import oracle
import paro_inputs as pin

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


def _random_operand(rng, rows, C, lo, hi):
    codes = rng.integers(0, 16, size=(rows, C), dtype=np.uint8)
    scales = rng.integers(lo, hi, size=(rows, C // 32), dtype=np.uint8)
    return codes, scales


def _words(codes):
    w = np.zeros((codes.shape[0], codes.shape[1] // 8), dtype=np.uint32)
    for k in range(8):
        w |= codes[:, k::8].astype(np.uint32) << np.uint32(4 * k)
    return w


def _allowed(xc, xs, wc, ws, y):
    C = xc.shape[1]
    mass = np.abs(oracle.mxfp4_dequant(xc, xs)) @ np.abs(oracle.mxfp4_dequant(wc, ws)).T
    return 2.0 ** -11 * np.abs(y) * 1.001 + (C / 128 + 16) * 2.0 ** -23 * mass + 2.0 ** -25


def _check(got, xc, xs, wc, ws, bias, label):
    y = oracle.mxfp4_linear(xc, xs, wc, ws, bias)
    worst = float((np.abs(got.astype(np.float64) - y) / _allowed(xc, xs, wc, ws, y)).max())
    say(f"  {label}: worst err/allowed = {worst:.3f} over {y.size} outputs, max |y| = {np.abs(y).max():.1f}")
    assert np.isfinite(got.astype(np.float32)).all()
    assert worst <= 1.0, label


@pytest.mark.parametrize("shape", [(48, 512), (16, 1024), (272, 4096), (32, 14336)])
def test_repack_and_unpack_are_bit_exact(P, shape):
    import torch
    N, C = shape
    rng = np.random.default_rng(9100 + N)
    wc, ws = _random_operand(rng, N, C, 0, 256)
    w = P.Mxfp4Weight.from_host(wc, ws)
    c0, s0 = P.paro_mxfp4_unpack(w)
    assert np.array_equal(c0.cpu().numpy(), wc) and np.array_equal(s0.cpu().numpy(), ws)
    P.paro_mxfp4_repack(w)
    w.c.codes = w.c.scales = None                       # only the blob from here
    c1, s1 = P.paro_mxfp4_unpack(w)
    torch.cuda.synchronize()
    assert np.array_equal(c1.cpu().numpy(), wc) and np.array_equal(s1.cpu().numpy(), ws)


@pytest.mark.parametrize("case", [
    dict(seed=9201, T=1, C=512, N=16, bias=False),
    dict(seed=9202, T=3, C=1024, N=48, bias=True),
    dict(seed=9203, T=16, C=4096, N=272, bias=True),          # 17 tiles: a ragged last block
    dict(seed=9204, T=5, C=14336, N=64, bias=False),          # 28 slices: 3 per wave
    dict(seed=9205, T=2, C=27648, N=32, bias=True),           # 54 slices: 5 per wave
    dict(seed=9206, T=37, C=1024, N=80, bias=True),           # three passes of up to 16 tokens
    dict(seed=9207, T=1, C=4096, N=6144, bias=False),         # more tiles than blocks
    dict(seed=9208, T=16, C=6144, N=4112, bias=False),        # 12 slices, 257 tiles
    dict(seed=9209, T=65, C=512, N=256, bias=True),           # tiled kernel from 65 tokens: one tile, 4 K-steps
    dict(seed=9210, T=300, C=1024, N=272, bias=True),         # ragged in tokens and in outputs
    dict(seed=9211, T=257, C=2048, N=528, bias=False),        # a second token tile of one row
    dict(seed=9212, T=1024, C=4096, N=1536, bias=True),       # 8 x 6 tiles of 128 tokens, 32 K-steps
    dict(seed=9221, T=2100, C=512, N=3856, bias=True),        # 9 x 16 tiles of 256 tokens (more than half a round), ragged both ways
    dict(seed=9222, T=2048, C=512, N=9216, bias=False),       # 8 x 36 = 288 tiles: one round of 256-token tiles, the last 4 output tiles as 128-token tiles
    dict(seed=9215, T=64, C=4096, N=528, bias=True),          # 64 tokens in one pass: four token blocks per wave
    dict(seed=9216, T=40, C=5120, N=272, bias=False),         # 10 slices, three of four token blocks used
    dict(seed=9217, T=32, C=14336, N=96, bias=True),          # 28 slices: 4 per wave, two token blocks
    dict(seed=9218, T=50, C=14336, N=48, bias=False),         # the same K: a pass of 32 and a pass of 18
    dict(seed=9219, T=20, C=27648, N=32, bias=False),         # 54 slices: 16 tokens per pass only (16 + 4)
    dict(seed=9220, T=48, C=8192, N=64, bias=True),           # 16 slices: 2 per wave, four token blocks
    dict(seed=9213, T=70, C=512, N=64, bias=True, pad=2),     # output rows that are not 16-byte aligned
    dict(seed=9214, T=3, C=512, N=48, bias=False, pad=6),
])
def test_mxfp4_linear_against_oracle(P, case):
    import torch
    say(f"mxfp4 linear {case}")
    rng = np.random.default_rng(case["seed"])
    T, C, N = case["T"], case["C"], case["N"]
    xc, xs = _random_operand(rng, T, C, 118, 128)
    wc, ws = _random_operand(rng, N, C, 113, 123)
    bias = rng.standard_normal(N).astype(np.float16) if case["bias"] else None
    w = P.Mxfp4Weight.from_host(wc, ws, bias)
    P.paro_mxfp4_repack(w)
    w.c.codes = w.c.scales = None
    x_codes = torch.as_tensor(_words(xc).view(np.int32)).cuda()
    x_scales = torch.as_tensor(xs).cuda()
    pad = case.get("pad", 0)
    Y = torch.full((T, N + pad), 7.0, dtype=torch.float16, device="cuda")
    got = P.paro_mxfp4_linear(w, x_codes, x_scales, Y[:, :N]).cpu().numpy()
    _check(got, xc, xs, wc, ws, bias, "every output")
    if pad:
        assert bool((Y[:, N:] == 7.0).all())                 # nothing written beyond a row's outputs


def test_zero_blocks_and_extreme_scales(P):
    """All-zero blocks (scale byte 0), -0 codes, and block scales 60 binades apart in one row."""
    import torch
    rng = np.random.default_rng(9301)
    T, C, N = 4, 1024, 32
    xc, xs = _random_operand(rng, T, C, 120, 126)
    wc, ws = _random_operand(rng, N, C, 120, 126)
    xc[:, 32:64] = 0; xs[:, 1] = 0
    wc[:, 96:128] = 8; ws[:, 3] = 0                      # -0 everywhere in the block
    xs[:, 4] = 97; ws[:, 4] = 157                        # tiny x block against a huge w block: product scale 2^0
    xs[1, 5] = 90                                        # a block 30+ binades below its neighbours
    w = P.Mxfp4Weight.from_host(wc, ws)
    P.paro_mxfp4_repack(w)
    got = P.paro_mxfp4_linear(w, torch.as_tensor(_words(xc).view(np.int32)).cuda(), torch.as_tensor(xs).cuda()).cpu().numpy()
    _check(got, xc, xs, wc, ws, None, "special blocks")


def test_weight_quantiser_without_rotation_is_bit_exact(P):
    """Q(W) with T = identity: fp16 inputs, power-of-two scaling and threshold compares are exact on both sides."""
    import torch
    rng = np.random.default_rng(9401)
    N, C = 40, 1024
    w16 = (rng.standard_normal((N, C)) * np.exp2(rng.integers(-6, 4, size=(N, 1)))).astype(np.float16)
    w16[3, 64:96] = 0
    w = P.paro_mxfp4_quantize_weight(None, torch.as_tensor(w16).cuda())
    codes, scales = P.paro_mxfp4_unpack(w)
    rc, rs = oracle.mxfp4_quantize(w16.astype(np.float64))
    assert np.array_equal(scales.cpu().numpy(), rs)
    got, ref = codes.cpu().numpy(), rc
    nz = (ref & 7) != 0
    assert np.array_equal(got & 7, ref & 7) and np.array_equal((got & 8)[nz], (ref & 8)[nz])


@pytest.mark.parametrize("case", [
    dict(seed=9501, T=1, c_in=512, c_out=64),
    dict(seed=9502, T=9, c_in=1024, c_out=144),
    dict(seed=9503, T=20, c_in=4096, c_out=96),
    dict(seed=9504, T=150, c_in=1024, c_out=304),             # tiled kernel
])
def test_whole_equation_from_dense_weight_and_fp16_activations(P, case):
    """Q(T W) on the GPU, Q(X T^-1) on the GPU inside paro_rotated_linear_mxfp4, then the contraction: the output must
    be the oracle's contraction of exactly the codes the two quantisers produced; the weight codes themselves are the
    oracle's fp64 transform + conversion except where the fp32 rotation crosses a decision threshold; and the result
    approximates the unquantised W x as 4-bit operands can."""
    import torch
    say(f"whole MXFP4 equation {case}")
    li = pin.make_custom(case["seed"], case["T"], case["c_in"], case["c_out"], n_outlier=3)
    rot = P.Rotation(li.pairs, li.theta, li.ch_scale)
    P.paro_rotation_plan_build(rot)
    rng = np.random.default_rng(case["seed"])
    w16 = (rng.standard_normal((case["c_out"], case["c_in"])) * 0.05).astype(np.float16)
    bias = rng.standard_normal(case["c_out"]).astype(np.float16)
    w = P.paro_mxfp4_quantize_weight(rot, torch.as_tensor(w16).cuda(), torch.as_tensor(bias).cuda())
    wc_t, ws_t = P.paro_mxfp4_unpack(w)
    wc, ws = wc_t.cpu().numpy(), ws_t.cpu().numpy()
    # weight side against the oracle
    wt = oracle.weight_transform(w16, li.pairs, li.theta, li.ch_scale)
    rc, rs = oracle.mxfp4_quantize(wt)
    de = ws.astype(np.int32) - rs.astype(np.int32)
    assert np.abs(de).max() <= 1 and (de != 0).mean() < 2e-3, (np.abs(de).max(), (de != 0).mean())
    same = np.repeat(de == 0, 32, axis=1)
    agree = ((wc & 7) == (rc & 7))[same].mean()
    say(f"  weight codes equal to the fp64 oracle's: {agree:.5f}")
    assert agree > 0.998
    # the call
    P.paro_mxfp4_repack(w)
    x = torch.as_tensor(li.x).cuda()
    ws_buf = torch.empty(P.paro_workspace_bytes_mxfp4(case["c_in"], case["T"]), dtype=torch.uint8, device="cuda")
    got = P.paro_rotated_linear_mxfp4(rot, w, x, ws_buf).cpu().numpy()
    xc_t, xs_t = P.paro_rotate_scale_quantize_mxfp4(rot, x)
    xc = oracle.unpack_codes(xc_t.cpu().numpy().view(np.uint32))
    xs = xs_t.cpu().numpy()
    _check(got, xc, xs, wc, ws, bias, "against the contraction of the GPU's own codes")
    exact = li.x.astype(np.float64) @ w16.astype(np.float64).T + bias.astype(np.float64)
    rel = np.linalg.norm(got.astype(np.float64) - exact) / np.linalg.norm(exact)
    say(f"  relative error against the unquantised W x + b: {rel:.3f}")
    assert rel < 0.35


def test_graph_replays_match_eager(P):
    """The MXFP4 calls only enqueue kernels: a captured sequence (whole equation at 3 tokens, contraction at 40 and at
    150 tokens) replays to the eager bits, with eager work between the replays."""
    import torch
    li = pin.make_custom(9601, 150, 1024, 176, n_outlier=3)
    rot = P.Rotation(li.pairs, li.theta, li.ch_scale)
    P.paro_rotation_plan_build(rot)
    rng = np.random.default_rng(9601)
    w = P.paro_mxfp4_quantize_weight(rot, torch.as_tensor((rng.standard_normal((176, 1024)) * 0.05).astype(np.float16)).cuda())
    P.paro_mxfp4_repack(w)
    x = torch.as_tensor(li.x).cuda()
    xc, xs = P.paro_rotate_scale_quantize_mxfp4(rot, x)
    buf = torch.empty(P.paro_workspace_bytes_mxfp4(1024, 3), dtype=torch.uint8, device="cuda")
    outs = [torch.zeros((t, 176), dtype=torch.float16, device="cuda") for t in (3, 40, 150)]

    def sequence():
        P.paro_rotated_linear_mxfp4(rot, w, x[:3], buf, Y=outs[0])
        P.paro_mxfp4_linear(w, xc[:40], xs[:40], outs[1])
        P.paro_mxfp4_linear(w, xc, xs, outs[2])

    sequence()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            sequence()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), rep
        sequence()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), rep
