"""GPU parity: the HIP path (through the C ABI binding) against the fp64 CPU oracle,
element by element, on seeded inputs.

  unpack / zero points / dequant : bit-exact
  rotated activations            : within 2 fp16 ulp (tests/paro_tol.py states the floor)
  linear outputs                 : |err| <= 5e-3 * ||w_row|| * ||u_t|| / sqrt(c_in)
"""
import sys

import numpy as np
import pytest

import oracle
import paro_inputs as pin
from paro_tol import linear_allowed, rotation_check

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2511_10645_amd as paro
    assert torch.cuda.is_available()
    paro.lib()
    return paro


def dev(a):
    import torch
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


def make_rot(P, li, plan=True, scale=True, scale_order=0):
    r = P.Rotation(li.pairs, li.theta, li.ch_scale if scale else None, scale_order=scale_order)
    if plan:
        P.paro_rotation_plan_build(r)
    return r


def make_w(P, li, packed=True, bias=None):
    w = P.W4Weight(li.qweight, li.scales, li.qzeros, bias=bias)
    if packed:
        P.paro_w4_repack(w)
    return w


# ----------------------------------------------------------------------------- bit-exact hooks

@pytest.mark.parametrize("shape", [(512, 512), (1024, 16 * 37), (1536, 48)])
def test_unpack_and_dequant_bit_exact(P, shape):
    c_in, c_out = shape
    say(f"hooks c_in={c_in} c_out={c_out}")
    li = pin.make_custom(100 + c_in, 1, c_in, c_out)
    want_codes = oracle.unpack_codes(li.qweight)
    want_zeros = oracle.unpack_zeros(li.qzeros)
    want_deq = oracle.round_fp16(oracle.dequant(li.qweight, li.scales, li.qzeros)).view(np.uint16)
    assert np.array_equal(want_codes, li.codes) and np.array_equal(want_zeros, li.zeros)
    for packed in (False, True):
        w = make_w(P, li, packed=packed)
        if packed:
            w.drop_interchange()        # the hooks must read the repacked blob, not the original
        assert np.array_equal(P.paro_w4_unpack_codes(w).cpu().numpy(), want_codes), f"codes packed={packed}"
        assert np.array_equal(P.paro_w4_unpack_zeros(w).cpu().numpy(), want_zeros), f"zeros packed={packed}"
        got = P.paro_w4_dequant(w).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want_deq), f"dequant packed={packed}"


def test_dequant_bit_exact_over_scale_range(P):
    """Scales across the whole fp16 range (subnormal products, large products)."""
    say("dequant scale sweep")
    rng = np.random.default_rng(77)
    li = pin.make_custom(78, 1, 512, 1024)
    bits = rng.integers(0, 0x7800, size=li.scales.shape).astype(np.uint16)       # finite, up to 2^15
    li.scales = bits.view(np.float16)
    want = oracle.round_fp16(oracle.dequant(li.qweight, li.scales, li.qzeros)).view(np.uint16)
    for packed in (False, True):
        w = make_w(P, li, packed=packed)
        assert np.array_equal(P.paro_w4_dequant(w).cpu().numpy().view(np.uint16), want)


# ----------------------------------------------------------------------------- rotation

def _check_rot(P, li, rot, ref, note, X=None):
    import torch
    x = dev(li.x) if X is None else X
    got = P.paro_rotate_scale(rot, x).cpu().numpy()
    ok, stats = rotation_check(got[:, :li.c_in], ref)
    say(f"{note}: {stats}")
    assert ok, (note, stats)
    return stats


@pytest.mark.parametrize("plan", [True, False])
def test_rotate_config0(P, plan):
    li = pin.make_linear(0, 0)
    ref = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    stats = _check_rot(P, li, make_rot(P, li, plan=plan), ref, f"rotate config0 plan={plan}")
    assert stats["frac_within_2ulp_strict"] > 0.98


@pytest.mark.parametrize("plan", [True, False])
@pytest.mark.parametrize("case", [
    dict(T=37, c_in=384, K=8, P=64, scale=True, order=0),
    dict(T=5, c_in=256, K=3, P=64, scale=True, order=1),
    dict(T=19, c_in=256, K=8, P=40, scale=False, order=0),
    dict(T=2, c_in=128, K=1, P=1, scale=True, order=0),
    dict(T=130, c_in=640, K=5, P=17, scale=True, order=1),
])
def test_rotate_edge_shapes(P, plan, case):
    li = pin.make_custom(500 + case["T"], case["T"], case["c_in"], 16, n_layers=case["K"],
                         pairs_per_layer=case["P"], n_outlier=2)
    cs = li.ch_scale if case["scale"] else None
    ref = oracle.rotate_scale(li.x, li.pairs, li.theta, cs, scale_order=case["order"])
    rot = make_rot(P, li, plan=plan, scale=case["scale"], scale_order=case["order"])
    _check_rot(P, li, rot, ref, f"rotate {case} plan={plan}")


def test_rotate_zero_layers_and_identity(P):
    li = pin.make_custom(9, 4, 256, 16)
    say("rotate K=0 / theta=0")
    import torch
    rot0 = P.Rotation(li.pairs[:, :0], li.theta[:, :0], li.ch_scale)
    P.paro_rotation_plan_build(rot0)
    ref = li.x.astype(np.float64) * li.ch_scale.astype(np.float64)
    got = P.paro_rotate_scale(rot0, dev(li.x)).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), oracle.round_fp16(ref).view(np.uint16))
    rot1 = P.Rotation(li.pairs, np.zeros_like(li.theta), None)
    P.paro_rotation_plan_build(rot1)
    got = P.paro_rotate_scale(rot1, dev(li.x)).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), li.x.view(np.uint16))       # identity transform is exact


def test_rotate_in_place_and_strided(P):
    import torch
    li = pin.make_custom(10, 33, 384, 16, n_outlier=3)
    ref = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    rot = make_rot(P, li)
    say("rotate in place, ld > c_in")
    buf = torch.zeros((33, 400), dtype=torch.float16, device="cuda")
    buf[:, :384] = dev(li.x)
    buf[:, 384:] = 7.0
    view = buf[:, :384]
    P.paro_rotate_scale(rot, view, view)
    got = buf.cpu().numpy()
    ok, stats = rotation_check(got[:, :384], ref)
    assert ok, stats
    assert (got[:, 384:] == 7.0).all()                                   # padding untouched


# ----------------------------------------------------------------------------- linear

def _linear_ref(li, u, bias=None):
    y = oracle.linear(u, li.qweight, li.scales, li.qzeros, bias)
    allowed = linear_allowed(oracle.row_sqnorms(li.qweight, li.scales, li.qzeros), u)
    return y, allowed


def _assert_linear(got16, y, allowed, note):
    err = np.abs(got16.astype(np.float64) - y)
    worst = float((err / allowed).max())
    say(f"{note}: worst err/allowed = {worst:.3f}")
    assert worst <= 1.0, (note, worst)
    return worst


@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("case", [
    dict(T=1, c_in=512, c_out=512),
    dict(T=3, c_in=1024, c_out=16 * 37),
    dict(T=16, c_in=1536, c_out=16 * 9),
    dict(T=23, c_in=2048, c_out=16 * 21),
    dict(T=300, c_in=1024, c_out=16 * 21),      # MFMA GEMM path, ragged token and output tiles
    dict(T=257, c_in=512, c_out=16 * 33),
    dict(T=17, c_in=1024, c_out=16 * 21),       # 17 tokens: one pass with a second, nearly empty block of 16 tokens
    dict(T=1, c_in=6144, c_out=16 * 37),        # 12 K-slices: the widest single-block reduction
    dict(T=5, c_in=6656, c_out=16 * 11),        # 13 K-slices: spread over two blocks of 7 waves, partials exchanged
    dict(T=16, c_in=5120, c_out=16 * 19),       # 10 K-slices, a full 16-token pass
    dict(T=300, c_in=512, c_out=16 * 1037),     # GEMM with 256 x 192 tiles (130 tiles of 256 x 256 would leave half the chip idle), ragged both ways
    dict(T=32, c_in=4096, c_out=16 * 37),       # one pass with two blocks of 16 tokens per wave
    dict(T=20, c_in=5120, c_out=16 * 19),       # 10 K-slices: two blocks of 5 waves in the two-block kernel, partials exchanged
    dict(T=29, c_in=6656, c_out=16 * 11),       # 13 K-slices, 29 tokens
    dict(T=31, c_in=512, c_out=16 * 700),       # more tiles than one round of blocks takes at 9 per block
    dict(T=50, c_in=1024, c_out=16 * 21),       # a pass of 32 and a pass of 18 tokens
])
def test_bare_linear(P, packed, case):
    li = pin.make_custom(700 + case["T"], case["T"], case["c_in"], case["c_out"], n_outlier=3)
    bias = pin.make_bias(9, 9, case["c_out"]) if case["T"] in (3, 5, 300, 29, 32) else None
    u = li.x.astype(np.float64)
    y, allowed = _linear_ref(li, u, bias)
    w = make_w(P, li, packed=packed, bias=bias)
    ws = P.Workspace(P.paro_workspace_bytes(None, w, case["T"]))
    got = P.paro_w4a16_linear(w, dev(li.x), ws).cpu().numpy()
    _assert_linear(got, y, allowed, f"bare {case} packed={packed}")
    ex = P.paro_workspace_exchange_bytes(None, w, case["T"])
    ws.exchange_bytes = ex                                              # 0: the buffer is scratch only, no header to read
    assert ws.partials_clean(ex) and ws.error_word() == 0               # partial sums left zero-filled


@pytest.mark.parametrize("case", [
    dict(T=1, c_in=512, c_out=512, plan=True, packed=True),
    dict(T=1, c_in=2048, c_out=16 * 37, plan=True, packed=True),
    dict(T=4, c_in=1024, c_out=16 * 13, plan=True, packed=True),
    dict(T=7, c_in=1024, c_out=16 * 13, plan=True, packed=True),
    dict(T=16, c_in=1536, c_out=256, plan=True, packed=True),
    dict(T=40, c_in=512, c_out=16 * 5, plan=True, packed=True),
    dict(T=4, c_in=6656, c_out=16 * 11, plan=True, packed=True),     # fused, 13 K-slices exchanged
    dict(T=5, c_in=6656, c_out=16 * 11, plan=True, packed=True),     # rotation pass + wide kernel over two blocks
    dict(T=16, c_in=6144, c_out=16 * 37, plan=True, packed=True),
    dict(T=2, c_in=1024, c_out=64, plan=False, packed=True),
    dict(T=2, c_in=640, c_out=64, plan=True, packed=False),
    dict(T=3, c_in=512, c_out=64, plan=False, packed=False),
])
def test_rotated_linear(P, case):
    li = pin.make_custom(900 + case["T"] + case["c_in"], case["T"], case["c_in"], case["c_out"], n_outlier=3)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    y, allowed = _linear_ref(li, u)
    rot = make_rot(P, li, plan=case["plan"])
    w = make_w(P, li, packed=case["packed"])
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, case["T"]))
    x = dev(li.x)
    got = P.paro_rotated_linear(rot, w, x, ws)
    _assert_linear(got.cpu().numpy(), y, allowed, f"rotated {case}")
    # same call again on the same workspace: bit-identical (deterministic reduction, clean counters)
    got2 = P.paro_rotated_linear(rot, w, x, ws)
    assert (got == got2).all()
    if case["T"] <= 4 and case["plan"] and case["packed"]:
        assert ws.partials_clean() and ws.error_word() == 0              # no partial sums left behind, no wait ran out


@pytest.mark.parametrize("T", [1, 3, 16, 27, 40, 300])
@pytest.mark.parametrize("fused", [False, True])
def test_linear_with_padded_rows(P, T, fused):
    """X and Y as column slices of wider buffers (ld > width): every kernel of the dispatch (narrow, wide,
    rotation pass, GEMM) must honour both strides and leave Y's padding columns alone."""
    import torch
    c_in, c_out = 1024, 16 * 21
    say(f"padded rows T={T} fused={fused}")
    li = pin.make_custom(5100 + T, T, c_in, c_out, n_outlier=3)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale) if fused else li.x.astype(np.float64)
    y, allowed = _linear_ref(li, u)
    w = make_w(P, li)
    rot = make_rot(P, li) if fused else None
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, T))
    xbuf = torch.full((T, c_in + 64), 3.0, dtype=torch.float16, device="cuda")
    xbuf[:, 8:8 + c_in] = dev(li.x)
    ybuf = torch.full((T, c_out + 24), 7.0, dtype=torch.float16, device="cuda")
    xv, yv = xbuf[:, 8:8 + c_in], ybuf[:, 16:16 + c_out]
    if fused:
        P.paro_rotated_linear(rot, w, xv, ws, Y=yv)
    else:
        P.paro_w4a16_linear(w, xv, ws, Y=yv)
    got = ybuf.cpu().numpy()
    _assert_linear(got[:, 16:16 + c_out], y, allowed, f"padded rows T={T} fused={fused}")
    assert (got[:, :16] == 7.0).all() and (got[:, 16 + c_out:] == 7.0).all()
    assert (xbuf[:, :8] == 3.0).all() and (xbuf[:, 8:8 + c_in].cpu().numpy() == li.x).all()          # input untouched


def test_pair_table_that_breaks_def1_gives_nan_on_both_paths(P):
    """A channel named twice in one layer (or an index outside the group) has no defined result: the affected
    group comes out as NaN with and without a plan, the other groups are untouched."""
    li = pin.make_custom(55, 3, 384, 64)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    bad = li.pairs.copy()
    bad[1, 2, 7, 1] = bad[1, 2, 9, 0]                                  # group 1, layer 2: a channel twice
    bad[2, 5, 0, 0] = 128                                              # group 2: index out of range
    assert P.paro_validate_pairs_host(bad) != 0
    for plan in (True, False):
        rot = P.Rotation(bad, li.theta, li.ch_scale)
        if plan:
            P.paro_rotation_plan_build(rot)
        got = P.paro_rotate_scale(rot, dev(li.x)).cpu().numpy()
        assert np.isnan(got[:, 128:384].astype(np.float32)).all(), plan
        ok, stats = rotation_check(got[:, :128], u[:, :128])
        assert ok, (plan, stats)


def test_graph_replays_match_eager(P):
    """The calls only enqueue kernels (no memset nodes, no allocation), so a captured sequence can be replayed:
    every replay, with eager work in between, must reproduce the eager bits and leave the workspace zero-filled."""
    import torch
    say("graph replays")
    li = pin.make_custom(77, 4, 2048, 16 * 37, n_outlier=3)
    lp = pin.make_custom(78, 40, 2048, 16 * 37, n_outlier=3)
    rot, w = make_rot(P, li), make_w(P, li)
    ws = P.Workspace.shared([(rot, w, 1), (rot, w, 4), (None, w, 4), (rot, w, 40)])
    x1, x4, x40 = dev(li.x[:1]), dev(li.x), dev(lp.x)
    outs = [torch.zeros((t, w.c_out), dtype=torch.float16, device="cuda") for t in (1, 4, 4, 40)]

    def sequence():
        P.paro_rotated_linear(rot, w, x1, ws, Y=outs[0])         # narrow kernel, split-K exchange
        P.paro_rotated_linear(rot, w, x4, ws, Y=outs[1])
        P.paro_w4a16_linear(w, x4, ws, Y=outs[2])                # wide kernel
        P.paro_rotated_linear(rot, w, x40, ws, Y=outs[3])        # rotation pass + GEMM or streamed passes

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
        assert ws.partials_clean(ws.exchange_bytes) and ws.error_word() == 0
        sequence()                                               # eager work between replays
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), rep


def test_long_strided_input_walked_in_runs(P):
    """Rows 4 MiB apart: 600 of them span more than the 31-bit offsets one GEMM launch addresses, so the
    call walks the tokens in runs of whole tiles (256 + 256 + 88 here); results as for any other input."""
    import torch
    T, c_in, c_out, ld = 600, 512, 16 * 21, 1 << 21
    say(f"long strided input T={T} ld={ld}")
    li = pin.make_custom(4242, T, c_in, c_out, n_outlier=3)
    y, allowed = _linear_ref(li, li.x.astype(np.float64))
    w = make_w(P, li)
    ws = P.Workspace(P.paro_workspace_bytes(None, w, T))
    big = torch.empty((T, ld), dtype=torch.float16, device="cuda")
    big[:, :c_in] = dev(li.x)
    got = P.paro_w4a16_linear(w, big[:, :c_in], ws).cpu().numpy()
    del big
    _assert_linear(got, y, allowed, "bare, long strided input")


def test_identity_transform_equals_bare_linear(P):
    """theta = 0 and scale = 1: the fused call must give the bare linear's bits."""
    li = pin.make_custom(31, 2, 1024, 256)
    say("identity transform")
    rot = P.Rotation(li.pairs, np.zeros_like(li.theta), None)
    P.paro_rotation_plan_build(rot)
    w = make_w(P, li)
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, 2))
    a = P.paro_rotated_linear(rot, w, dev(li.x), ws)
    b = P.paro_w4a16_linear(w, dev(li.x), ws)
    assert (a == b).all()


# ----------------------------------------------------------------------------- full configs

def _column_subset(li, cols):
    """The linear restricted to the output columns `cols` (a multiple of 8 of them), interchange layout."""
    z = oracle.unpack_zeros(li.qzeros)[:, cols]
    return np.ascontiguousarray(li.qweight[cols]), np.ascontiguousarray(li.scales[:, cols]), pin.pack_nibbles_u32(z)


def _check_block(got, u, qw, sc, qz, c_in, label):
    """Every element of `got` ([rows of u] x [all columns of the given weight]) against the oracle."""
    y = oracle.linear(u, qw, sc, qz)
    allowed = linear_allowed(oracle.row_sqnorms(qw, sc, qz), u)
    worst = float((np.abs(got.astype(np.float64) - y) / allowed).max())
    say(f"  {label}: worst err/allowed = {worst:.3f} over {y.size} outputs")
    assert worst <= 1.0, label


def _full_config_case(P, config, linear, T, n_samples=4096):
    """Full-size check in the launch configuration the benchmark times.  Rotation: every element against the
    oracle, and the strict 2-ulp statistic.  Linear outputs: up to 32 tokens EVERY output; beyond that whole stripes
    (all outputs of the first and the last 32 tokens; all tokens of 256 output columns: the first 64, the last 128 -
    the last output tile and the separately launched tail - and 64 spread over the middle) plus random samples."""
    li = pin.make_linear(config, linear, tokens=T, keep_codes=False)
    say(f"config {config} {li.shape.name} T={T} C={li.c_in} N={li.c_out}")
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    rot, w = make_rot(P, li), make_w(P, li)
    x = dev(li.x)
    xr = P.paro_rotate_scale(rot, x).cpu().numpy()
    ok, stats = rotation_check(xr, u)
    say(f"  rotation {stats}")
    assert ok, stats
    assert stats["frac_within_2ulp_strict"] >= 0.9999, stats
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, T))
    w.drop_interchange()
    got = P.paro_rotated_linear(rot, w, x, ws).cpu().numpy()
    assert np.isfinite(got.astype(np.float32)).all()
    # the bare linear on the rotated fp16 activations (oracle fed with those bits)
    yb = P.paro_w4a16_linear(w, dev(xr), ws).cpu().numpy()
    ub = xr.astype(np.float64)
    assert ws.error_word() == 0
    if T <= 32:
        _check_block(got, u, li.qweight, li.scales, li.qzeros, li.c_in, "fused, every output")
        _check_block(yb, ub, li.qweight, li.scales, li.qzeros, li.c_in, "bare, every output")
        two_launches = P.paro_workspace_bytes(rot, w, T) > P.paro_workspace_exchange_bytes(rot, w, T)
        if T <= 4 and two_launches:
            # the call preferred rotation pass + bare kernel on this shape; the kernel that hosts the rotation is
            # still reachable through the entry point without a workspace, where its exchange part fits that array
            import torch
            yn = torch.full((T, li.c_out), float("nan"), dtype=torch.float16, device="cuda")
            rc = P.lib().paro_rotated_linear_noalloc(rot.ref(), w.ref(), x.data_ptr(), x.stride(0), yn.data_ptr(),
                                                     yn.stride(0), T, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            say(f"  two-launch shape; fused kernel through the no-workspace entry: rc = {rc}")
            assert rc in (0, 6)
            if rc == 0:
                _check_block(yn.cpu().numpy(), u, li.qweight, li.scales, li.qzeros, li.c_in, "fused kernel, every output")
        return
    rows = np.r_[0:32, T - 32:T]
    _check_block(got[rows], u[rows], li.qweight, li.scales, li.qzeros, li.c_in, "fused, all outputs of 64 tokens")
    _check_block(yb[rows], ub[rows], li.qweight, li.scales, li.qzeros, li.c_in, "bare, all outputs of 64 tokens")
    N = li.c_out
    cols = np.unique(np.r_[0:64, N - 128:N, np.linspace(64, N - 129, 64).astype(np.int64)])
    cols = cols[: len(cols) // 8 * 8]
    qw, sc, qz = _column_subset(li, cols)
    _check_block(got[:, cols], u, qw, sc, qz, li.c_in, f"fused, all tokens of {len(cols)} columns")
    _check_block(yb[:, cols], ub, qw, sc, qz, li.c_in, f"bare, all tokens of {len(cols)} columns")
    rng = np.random.default_rng(config * 10 + linear)
    ns = min(n_samples, T * li.c_out)
    t_idx = rng.integers(0, T, ns)
    n_idx = rng.integers(0, li.c_out, ns)
    ys, ww = oracle.linear_samples(u, li.qweight, li.scales, li.qzeros, t_idx, n_idx)
    allowed = 5e-3 * np.sqrt(ww) * np.linalg.norm(u, axis=1)[t_idx] / np.sqrt(li.c_in)
    worst = float((np.abs(got[t_idx, n_idx].astype(np.float64) - ys) / allowed).max())
    say(f"  fused, {ns} random samples: worst err/allowed = {worst:.3f}")
    assert worst <= 1.0


@pytest.mark.parametrize("linear", [0, 1, 2, 3])
def test_config1_decode_b1(P, linear):
    _full_config_case(P, 1, linear, 1)


@pytest.mark.parametrize("linear", [0, 1, 2, 3])
def test_config2_decode_b16(P, linear):
    _full_config_case(P, 2, linear, 16)


@pytest.mark.parametrize("linear", [0, 1, 2, 3])
def test_config3_prefill_2048(P, linear):
    _full_config_case(P, 3, linear, 2048)


@pytest.mark.parametrize("linear", [0, 1, 2, 3])
@pytest.mark.parametrize("T", [1, 4096])
def test_config4_32b(P, linear, T):
    _full_config_case(P, 4, linear, T)


@pytest.mark.parametrize("linear,T", [(0, 40), (1, 128), (2, 96), (3, 256), (3, 512), (2, 32), (3, 24)])
def test_config1_shapes_between_decode_and_prefill(P, linear, T):
    """Tens to hundreds of tokens on the 8B-class shapes: repeated streaming passes, or the GEMM with K split
    over blockIdx.y and the separate reduction, whichever the call picks."""
    _full_config_case(P, 1, linear, T)


def test_config0_tiny_full(P):
    li = pin.make_linear(0, 0)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    y, allowed = _linear_ref(li, u)
    rot, w = make_rot(P, li), make_w(P, li)
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, 1))
    got = P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy()
    _assert_linear(got, y, allowed, "config0 fused")


def test_one_workspace_shared_by_many_calls(P):
    """A model allocates one workspace and runs every linear through it.  The split-K exchange
    leaves it clean after each call, whatever shape, token count or path came before."""
    import torch
    say("shared workspace sequence")
    cases = []
    for seed, (T, c_in, c_out) in enumerate([(1, 2048, 16 * 50), (4, 1024, 16 * 13), (1, 6656, 16 * 11), (16, 1536, 256),
                                             (2, 512, 512), (7, 6656, 16 * 11), (1, 1024, 64), (40, 512, 16 * 5)]):
        li = pin.make_custom(1200 + seed, T, c_in, c_out, n_outlier=2)
        u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
        y_rot, allowed_rot = _linear_ref(li, u)
        y_bare, allowed_bare = _linear_ref(li, li.x.astype(np.float64))
        cases.append(dict(T=T, li=li, rot=make_rot(P, li), w=make_w(P, li), x=dev(li.x),
                          y_rot=y_rot, a_rot=allowed_rot, y_bare=y_bare, a_bare=allowed_bare))
    ws = P.Workspace.shared([(c["rot"], c["w"], c["T"]) for c in cases] + [(None, c["w"], c["T"]) for c in cases])
    assert ws.exchange_bytes > 0 and ws.nbytes > ws.exchange_bytes
    rs = np.random.default_rng(77)
    for it in range(60):
        c = cases[int(rs.integers(len(cases)))]
        if rs.integers(2):
            got = P.paro_rotated_linear(c["rot"], c["w"], c["x"], ws).cpu().numpy()
            _assert_linear(got, c["y_rot"], c["a_rot"], f"seq {it} rotated T={c['T']} C={c['li'].c_in}")
        else:
            got = P.paro_w4a16_linear(c["w"], c["x"], ws).cpu().numpy()
            _assert_linear(got, c["y_bare"], c["a_bare"], f"seq {it} bare T={c['T']} C={c['li'].c_in}")
        # the part every later call may use for its exchange is zero again, whatever ran (a separate
        # rotation pass leaves its output in the scratch part at the end of the buffer only)
        assert ws.partials_clean(ws.exchange_bytes) and ws.error_word() == 0, it
    torch.cuda.synchronize()


@pytest.mark.parametrize("case", [
    dict(T=1, c_in=1024, c_out=16 * 13, K=8, ppl=64, order=1),      # scale after the rotation
    dict(T=3, c_in=512, c_out=64, K=3, ppl=17, order=0),            # few layers, partial matchings, sentinels
    dict(T=2, c_in=1024, c_out=128, K=0, ppl=1, order=0),           # no rotation layer: scaling only
    dict(T=12, c_in=1024, c_out=16 * 13, K=5, ppl=40, order=1),     # unfused path (rotation pass + wide kernel)
])
def test_rotated_linear_transform_variants(P, case):
    li = pin.make_custom(1500 + case["K"] + case["T"], case["T"], case["c_in"], case["c_out"], n_layers=case["K"],
                         pairs_per_layer=case["ppl"], n_outlier=2)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=case["order"])
    y, allowed = _linear_ref(li, u)
    rot = make_rot(P, li, scale_order=case["order"])
    w = make_w(P, li)
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, case["T"]))
    got = P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy()
    _assert_linear(got, y, allowed, f"variants {case}")


def test_selected_pairs_through_the_gpu_path(P):
    """Algorithm A1's pairs (host) -> plan -> GPU rotation and fused linear, against the oracle."""
    say("pair selection end to end")
    c_in, c_out, T, K = 512, 16 * 9, 2, 8
    G = c_in // 128
    pairs = np.stack([P.paro_select_pairs_host(pin.make_pair_order(1600 + g), 128, K, 64)[0] for g in range(G)])
    li = pin.make_custom(1601, T, c_in, c_out)
    assert P.paro_validate_pairs_host(pairs) == 0
    rot = P.Rotation(pairs, li.theta, li.ch_scale)
    P.paro_rotation_plan_build(rot)
    ref = oracle.rotate_scale(li.x, pairs, li.theta, li.ch_scale)
    got = P.paro_rotate_scale(rot, dev(li.x)).cpu().numpy()
    ok, stats = rotation_check(got, ref)
    assert ok, stats
    y = oracle.linear(ref, li.qweight, li.scales, li.qzeros)
    allowed = linear_allowed(oracle.row_sqnorms(li.qweight, li.scales, li.qzeros), ref)
    w = make_w(P, li)
    ws = P.Workspace(P.paro_workspace_bytes(rot, w, T))
    _assert_linear(P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy(), y, allowed, "selected pairs")


def test_one_k_slice_with_a_very_wide_output(P):
    """512 input channels (one K-slice: nothing to exchange between blocks) against 98304 outputs (24 MB of codes, the
    size class that otherwise takes the 8-wave split-K blocks): the workspace holds the header only, and the guard
    bytes placed behind it must stay untouched."""
    import torch
    li = pin.make_custom(7901, 1, 512, 98304, n_outlier=2)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    y, allowed = _linear_ref(li, u)
    rot, w = make_rot(P, li), make_w(P, li)
    need = P.paro_workspace_bytes(rot, w, 1)
    assert need == P.paro_workspace_exchange_bytes(rot, w, 1) == 256
    guard = 1 << 20
    ws = P.Workspace(need + guard)
    ws.buf[need:] = 0x5A
    ws.nbytes = need
    got = P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy()
    _assert_linear(got, y, allowed, "one K-slice, 98304 outputs")
    assert bool((ws.buf[need:need + guard] == 0x5A).all())
    assert ws.error_word() == 0


@pytest.mark.parametrize("case", [(5, 1024, 53248), (16, 1536, 57344), (2, 6144, 45056), (9, 5120, 55296)],
                         ids=lambda c: f"T{c[0]}_{c[1]}to{c[2]}")
def test_long_streams_at_several_tokens(P, case):
    """Outputs wide enough that a block of the streaming kernel runs 11..14 tiles per wave at 2..16 tokens (1 KB of
    partial sums per tile and wave: the longest streams the LDS holds for 2, 3, 10 and 12 waves per block), bare and
    behind the rotation pass; every output is compared."""
    T, c_in, c_out = case
    li = pin.make_custom(7950 + T, T, c_in, c_out, n_outlier=2)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
    y, allowed = _linear_ref(li, u)
    yb, allowed_b = _linear_ref(li, li.x.astype(np.float64))
    rot, w = make_rot(P, li), make_w(P, li)
    ws = P.Workspace.shared([(rot, w, T), (None, w, T)])
    x = dev(li.x)
    _assert_linear(P.paro_w4a16_linear(w, x, ws).cpu().numpy(), yb, allowed_b, f"long stream bare {case}")
    _assert_linear(P.paro_rotated_linear(rot, w, x, ws).cpu().numpy(), y, allowed, f"long stream fused {case}")
    assert ws.partials_clean(ws.exchange_bytes) and ws.error_word() == 0


@pytest.mark.parametrize("case", [
    dict(c_in=512, c_out=163856, ppl=64, order=0, bias=False),      # one K-slice: blocks of one wave, a ragged last block
    dict(c_in=6144, c_out=24592, ppl=23, order=1, bias=True),       # 12 slices in one block, 7 tiles per wave; partial matchings, scale after
    dict(c_in=7168, c_out=11728, ppl=64, order=0, bias=True),       # 14 slices: two blocks of 7 waves per row, partial sums exchanged
    dict(c_in=1024, c_out=81936, ppl=64, order=0, bias=False, scale=False),   # two slices, no channel scale
], ids=lambda c: f"{c['c_in']}to{c['c_out']}")
def test_one_token_transform_inside_the_streaming_kernel(P, case):
    """One token and at least 4 tiles per wave (6 in blocks of more than 8 waves): the fused call runs the streaming kernel whose waves each
    transform their own K-slice from the compact plan (angles in 2^-24 revolutions, fp16 scales).  Every output
    against the oracle, on block shapes the benchmark configurations do not have; nothing but the header and the
    partial sums of a split row may be needed in the workspace."""
    c_in, c_out = case["c_in"], case["c_out"]
    li = pin.make_custom(7960 + c_in // 512, 1, c_in, c_out, pairs_per_layer=case["ppl"], n_outlier=2)
    bias = pin.make_bias(7960, 3, c_out) if case["bias"] else None
    scale = case.get("scale", True)
    u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale if scale else None, scale_order=case["order"])
    y, allowed = _linear_ref(li, u, bias)
    rot = make_rot(P, li, scale=scale, scale_order=case["order"])
    w = make_w(P, li, bias=bias)
    need = P.paro_workspace_bytes(rot, w, 1)
    assert need == P.paro_workspace_exchange_bytes(rot, w, 1) == max(256, P.paro_workspace_exchange_bytes(None, w, 1))
    ws = P.Workspace(need)
    got = P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy()
    _assert_linear(got, y, allowed, f"transform inside the streaming kernel {case}")
    assert ws.partials_clean() and ws.error_word() == 0
    # the same call twice more on the same workspace (the exchange part must come back empty)
    for _ in range(2):
        again = P.paro_rotated_linear(rot, w, dev(li.x), ws).cpu().numpy()
        assert np.array_equal(again.view(np.uint16), got.view(np.uint16)) or case["c_in"] > 6144
    # a pair table that breaks Def. 1 in one group has no defined result: every output becomes NaN on this path too
    bad = li.pairs.copy()
    bad[0, 3, 5, 1] = bad[0, 3, 6, 0]
    rot_bad = P.Rotation(bad, li.theta, li.ch_scale if scale else None, scale_order=case["order"])
    P.paro_rotation_plan_build(rot_bad)
    nan = P.paro_rotated_linear(rot_bad, w, dev(li.x), ws).cpu().numpy()
    assert np.isnan(nan.astype(np.float32)).all()


@pytest.mark.parametrize("ppl,order", [(64, 0), (23, 1), (1, 0)])
def test_compact_plan_rows_rotate_like_the_oracle(P, ppl, order):
    """The plan's compact copy read back and run in numpy, lane by lane: per group the channel ids and fp16 scales,
    per layer one angle (2^-24 revolutions) and the lane to pull from, `keep = cos A - sin B`, `send = cos B + sin A`
    with no case distinction.  It must reproduce the oracle's rotation (Eq. 4, 5, 8) to the accuracy of the angle
    grid: this pins the layout and the sign tracking of the plan builder apart from any kernel that reads it."""
    K, G = 8, 3
    li = pin.make_custom(7990 + ppl, 2, 128 * G, 16, pairs_per_layer=ppl)
    rot = make_rot(P, li, scale_order=order)
    words = rot.plan.cpu().numpy().view(np.uint32)
    compact = words[G * (5 + 3 * K) * 64:][:G * (3 + K) * 64].reshape(G, 3 + K, 64)
    x = li.x.astype(np.float64)
    ref = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=order)
    got = np.zeros_like(ref)
    h16 = lambda u: (u & 0xffff).astype(np.uint16).view(np.float16).astype(np.float64)
    for g in range(G):
        io, sci, sco = compact[g, 0], compact[g, 1], compact[g, 2]
        in_a, in_b, out_a, out_b = io & 0xff, (io >> 8) & 0xff, (io >> 16) & 0xff, io >> 24
        assert sorted(np.r_[in_a, in_b]) == list(range(128)) and sorted(np.r_[out_a, out_b]) == list(range(128))
        for t in range(x.shape[0]):
            row = x[t, g * 128:(g + 1) * 128]
            A, B = row[in_a] * h16(sci), row[in_b] * h16(sci >> 16)
            for l in range(K):
                m = compact[g, 3 + l]
                phi = 2.0 * np.pi * (m >> 8).astype(np.float64) / 2.0 ** 24
                src = (m & 0xff) >> 2
                keep, send = np.cos(phi) * A - np.sin(phi) * B, np.cos(phi) * B + np.sin(phi) * A
                A, B = keep, (send[src] if l + 1 < K else send)
            out = np.empty(128)
            out[out_a], out[out_b] = A * h16(sco), B * h16(sco >> 16)
            got[t, g * 128:(g + 1) * 128] = out
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max() / scale
    say(f"compact plan, {ppl} pairs per layer, scale order {order}: max error / max |x'| = {err:.2e}")
    assert err < 4e-6            # 8 layers x half a step of the angle grid (1.9e-7 rad), with margin


def test_seeded_sweep_of_shapes(P):
    """48 seeded draws of (T, c_in, c_out, layers, pairs per layer, scale order, bias, plan, repack): whatever
    kernel the dispatch picks (narrow, wide with 1..n blocks per column, rotation pass, GEMM with ragged tiles,
    interchange-layout fallback), the fused call and the bare call meet the linear gate."""
    rs = np.random.default_rng(20251127)
    for it in range(48):
        T = int(rs.choice([1, 2, 3, 4, 5, 9, 16, 17, 31, 64, 130, 257]))
        c_in = int(rs.choice([128, 384, 512, 1024, 1536, 2560, 4608, 7168]))
        c_out = 16 * int(rs.integers(1, 70))
        K = int(rs.choice([0, 1, 5, 8]))
        ppl = int(rs.choice([1, 23, 64]))
        order = int(rs.integers(2))
        plan, packed, with_bias = bool(rs.integers(4)), bool(rs.integers(4)), bool(rs.integers(2))
        packed = packed and c_in % 512 == 0                  # the repacked layout tiles K in slices of 4 groups
        case = dict(it=it, T=T, c_in=c_in, c_out=c_out, K=K, ppl=ppl, order=order, plan=plan, packed=packed, bias=with_bias)
        say(f"sweep {case}")
        li = pin.make_custom(7000 + it, T, c_in, c_out, n_layers=K, pairs_per_layer=ppl, n_outlier=2)
        bias = pin.make_bias(7000 + it, 3, c_out) if with_bias else None
        u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale, scale_order=order)
        y, allowed = _linear_ref(li, u, bias)
        yb, allowed_b = _linear_ref(li, li.x.astype(np.float64), bias)
        rot = make_rot(P, li, plan=plan, scale_order=order)
        w = make_w(P, li, packed=packed, bias=bias)
        ws = P.Workspace.shared([(rot, w, T), (None, w, T)])
        x = dev(li.x)
        _assert_linear(P.paro_rotated_linear(rot, w, x, ws).cpu().numpy(), y, allowed, f"sweep fused {case}")
        _assert_linear(P.paro_w4a16_linear(w, x, ws).cpu().numpy(), yb, allowed_b, f"sweep bare {case}")
        assert ws.partials_clean(ws.exchange_bytes) and ws.error_word() == 0, case
