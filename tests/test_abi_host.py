"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2511_10645_amd as paro
from paper_2511_10645_amd import binding as B
import paro_inputs as pin

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-NULL, 256-byte aligned; never dereferenced because validation fails first

(OK, E_NULL, E_SHAPE, E_ALIGN, E_PAIRS, E_UNSUP, E_WS, E_HIP) = range(8)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "paro.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(paro_[a-z0-9_]+)\s*\(", hdr)))
    assert len(names) >= 14
    L = ctypes.CDLL(paro.lib_path())
    for n in names:
        assert hasattr(L, n), n
    assert paro.paro_version() >= 100
    assert "Def. 1" in paro.paro_status_string(E_PAIRS)


def test_validate_pairs_host():
    li = pin.make_linear(0, 0)
    assert paro.paro_validate_pairs_host(li.pairs) == OK
    dup = li.pairs.copy(); dup[1, 3, 5, 1] = dup[1, 3, 9, 0]
    assert paro.paro_validate_pairs_host(dup) == E_PAIRS
    oob = li.pairs.copy(); oob[0, 0, 0, 0] = 128
    assert paro.paro_validate_pairs_host(oob) == E_PAIRS
    neg = li.pairs.copy(); neg[0, 0, 0, 1] = -1
    assert paro.paro_validate_pairs_host(neg) == E_PAIRS
    # empty slots (i, i) name no channel, even when repeated
    sent = li.pairs.copy(); sent[:, :, -2:, 1] = sent[:, :, -2:, 0]; sent[:, :, -1, :] = sent[:, :, -2, :]
    assert paro.paro_validate_pairs_host(sent) == OK
    assert paro.lib().paro_validate_pairs_host(None, 1, 1, 1, 128) == E_NULL


def _rot(**kw):
    d = dict(c_in=512, group=128, n_layers=8, pairs_per_layer=64, pairs=FAKE, theta=FAKE, ch_scale=FAKE,
             scale_order=0, plan=None)
    d.update(kw)
    return B._CRotation(**d)


def _w(**kw):
    d = dict(c_in=512, c_out=512, group=128, qweight=FAKE, scales=FAKE, qzeros=FAKE, bias=None, packed=None)
    d.update(kw)
    return B._CW4Weight(**d)


def test_rotate_scale_argument_errors():
    L = paro.lib()
    call = lambda r, X=FAKE, ldx=512, Xr=FAKE, ldxr=512, T=1: L.paro_rotate_scale(ctypes.byref(r), X, ldx, Xr, ldxr, T, None)
    assert L.paro_rotate_scale(None, FAKE, 512, FAKE, 512, 1, None) == E_NULL
    assert call(_rot(group=64)) == E_UNSUP
    assert call(_rot(n_layers=9)) == E_UNSUP
    assert call(_rot(pairs_per_layer=65)) == E_UNSUP
    assert call(_rot(scale_order=2)) == E_UNSUP
    assert call(_rot(c_in=500)) == E_SHAPE
    assert call(_rot(pairs=None)) == E_NULL
    assert call(_rot(), X=None) == E_NULL
    assert call(_rot(), T=0) == E_SHAPE
    assert call(_rot(), ldx=256) == E_SHAPE
    assert call(_rot(), ldx=513) == E_ALIGN
    assert call(_rot(), X=FAKE + 2) == E_ALIGN
    assert call(_rot(plan=FAKE + 16)) == E_ALIGN
    assert call(_rot(), Xr=FAKE, X=FAKE, ldx=512, ldxr=520) == E_SHAPE     # in place needs equal strides


def test_linear_argument_errors_and_workspace():
    L = paro.lib()
    lin = lambda w, X=FAKE, ldx=512, Y=FAKE, ldy=512, T=1, ws=None, n=0: L.paro_w4a16_linear(
        ctypes.byref(w), X, ldx, Y, ldy, T, ws, n, None)
    assert lin(_w(group=32)) == E_UNSUP
    assert lin(_w(c_out=520)) == E_SHAPE
    assert lin(_w(c_in=640 + 64)) == E_SHAPE
    assert lin(_w(qweight=None)) == E_NULL
    assert lin(_w(), Y=None) == E_NULL
    assert lin(_w(), ldy=256) == E_SHAPE
    assert lin(_w(), ldx=516) == E_ALIGN
    assert lin(_w(qweight=FAKE + 4)) == E_ALIGN
    # a repacked weight needs no workspace for the bare linear up to 6144 channels (all K-slices in one block) ...
    w2 = _w(c_in=1024, packed=FAKE)
    assert L.paro_workspace_bytes(None, ctypes.byref(w2), 1) == 0
    # ... and the partial sums of its blocks along K beyond that
    w3 = _w(c_in=14336, packed=FAKE)
    need = L.paro_workspace_bytes(None, ctypes.byref(w3), 1)
    assert need >= 256 + 4 * 1 * 512 * 4
    assert lin(w3, ldx=14336) == E_WS
    assert lin(w3, ldx=14336, ws=FAKE, n=need - 1) == E_WS
    rl = lambda r, w, ws=FAKE, n=1 << 30: L.paro_rotated_linear(ctypes.byref(r), ctypes.byref(w), FAKE, 1024, FAKE, 512, 1, ws, n, None)
    assert rl(_rot(c_in=512), w2) == E_SHAPE                       # rot.c_in != w.c_in
    assert rl(_rot(c_in=1024), w2, ws=None, n=0) == E_WS
    need_r = L.paro_workspace_bytes(ctypes.byref(_rot(c_in=1024)), ctypes.byref(w2), 3)
    assert need_r >= L.paro_workspace_bytes(None, ctypes.byref(w2), 3) + 3 * 1024 * 2
    assert L.paro_workspace_bytes(ctypes.byref(_rot(c_in=512)), ctypes.byref(w2), 1) == 0


def test_prepare_calls_argument_errors():
    L = paro.lib()
    # per group 5 + 3 K rows of 64 dwords, and the compact copy of 3 + K rows
    assert L.paro_rotation_plan_bytes(ctypes.byref(_rot())) == 4 * ((5 + 3 * 8) + (3 + 8)) * 64 * 4
    assert L.paro_rotation_plan_bytes(ctypes.byref(_rot(group=100))) == 0
    assert L.paro_rotation_plan_build(ctypes.byref(_rot()), None, None) == E_NULL
    assert L.paro_rotation_plan_build(ctypes.byref(_rot()), FAKE + 8, None) == E_ALIGN
    assert L.paro_w4_repack_bytes(ctypes.byref(_w())) == 32 * 4 * 1024 + 32 * 1 * 128 + 32 * 1 * 32
    assert L.paro_w4_repack_bytes(ctypes.byref(_w(c_in=640))) == 0      # 5 groups: not whole 512-channel slices
    assert L.paro_w4_repack(ctypes.byref(_w(c_in=640)), FAKE, None) == E_UNSUP
    assert L.paro_w4_repack(ctypes.byref(_w(qweight=None, packed=FAKE)), FAKE, None) == E_NULL
    assert L.paro_w4_unpack_codes(ctypes.byref(_w()), None, None) == E_NULL
    assert L.paro_w4_dequant(ctypes.byref(_w()), FAKE + 2, None) == E_ALIGN


def test_quantize_argument_errors():
    L = paro.lib()
    qz = lambda rot=None, W=FAKE, ldw=512, c_in=512, c_out=64, qw=FAKE, sc=FAKE, z=FAKE: L.paro_w4_quantize(
        None if rot is None else ctypes.byref(rot), W, ldw, c_in, c_out, qw, sc, z, None)
    assert qz(W=None) == E_NULL
    assert qz(qw=None) == E_NULL
    assert qz(c_in=500) == E_SHAPE
    assert qz(c_out=60) == E_SHAPE
    assert qz(ldw=256) == E_SHAPE
    assert qz(ldw=513) == E_ALIGN
    assert qz(W=FAKE + 2) == E_ALIGN
    assert qz(rot=_rot(c_in=1024)) == E_SHAPE            # rot.c_in != c_in
    assert qz(rot=_rot()) == E_UNSUP                      # a rotation without its plan
    assert qz(rot=_rot(n_layers=9)) == E_UNSUP


def test_multi_argument_errors():
    L = paro.lib()
    r1, r2 = _rot(c_in=1024), _rot(c_in=1024)
    w1, w2 = _w(c_in=1024, packed=FAKE), _w(c_in=1024, c_out=64, packed=FAKE)
    RA = (ctypes.c_void_p * 2)(ctypes.addressof(r1), ctypes.addressof(r2))
    WA = (ctypes.c_void_p * 2)(ctypes.addressof(w1), ctypes.addressof(w2))
    YA = (ctypes.c_void_p * 2)(FAKE, FAKE)
    LD = (ctypes.c_int64 * 2)(512, 64)
    L.paro_workspace_bytes_multi.restype = ctypes.c_size_t
    L.paro_workspace_bytes_multi.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
    need = L.paro_workspace_bytes_multi(2, RA, WA, 1)
    single = max(L.paro_workspace_bytes(ctypes.byref(r1), ctypes.byref(w1), 1), L.paro_workspace_bytes(ctypes.byref(r2), ctypes.byref(w2), 1))
    assert need >= single > 0
    call = lambda n=2, ra=RA, wa=WA, X=FAKE, ya=YA, ld=LD, T=1, ws=FAKE, nbytes=1 << 30: L.paro_rotated_linear_multi(
        n, ra, wa, X, 1024, ya, ld, T, ws, nbytes, None)
    assert call(n=0) == E_SHAPE
    assert call(n=5) == E_SHAPE
    assert call(ra=None) == E_NULL
    assert call(ya=None) == E_NULL
    assert call(ws=None, nbytes=0) == E_WS
    assert call(nbytes=need - 1) == E_WS
    r3 = _rot(c_in=512)
    RB = (ctypes.c_void_p * 2)(ctypes.addressof(r1), ctypes.addressof(r3))
    assert call(ra=RB) == E_SHAPE                                   # a part whose rotation does not fit its weight
    w3 = _w(c_in=512, packed=FAKE)
    WB = (ctypes.c_void_p * 2)(ctypes.addressof(w1), ctypes.addressof(w3))
    assert call(ra=RB, wa=WB) == E_SHAPE                            # parts with different c_in
    assert L.paro_workspace_bytes_multi(2, RB, WB, 1) == 0


def test_activation_quantize_argument_errors():
    L = paro.lib()
    q = lambda r, X=FAKE, ldx=512, T=1, c=FAKE, s=FAKE, z=FAKE: L.paro_rotate_scale_quantize_int4(
        ctypes.byref(r), X, ldx, T, c, s, z, None)
    assert L.paro_rotate_scale_quantize_int4(None, FAKE, 512, 1, FAKE, FAKE, FAKE, None) == E_NULL
    assert q(_rot(), X=None) == E_NULL
    assert q(_rot(), z=None) == E_NULL
    assert q(_rot(), T=0) == E_SHAPE
    assert q(_rot(), ldx=256) == E_SHAPE
    assert q(_rot(), ldx=513) == E_ALIGN
    assert q(_rot()) == E_UNSUP                       # no plan
    assert q(_rot(n_layers=9, plan=FAKE)) == E_UNSUP


def test_activation_mxfp4_argument_errors():
    L = paro.lib()
    q = lambda r, X=FAKE, ldx=512, T=1, c=FAKE, s=FAKE: L.paro_rotate_scale_quantize_mxfp4(
        ctypes.byref(r), X, ldx, T, c, s, None)
    assert L.paro_rotate_scale_quantize_mxfp4(None, FAKE, 512, 1, FAKE, FAKE, None) == E_NULL
    assert q(_rot(), X=None) == E_NULL
    assert q(_rot(), s=None) == E_NULL
    assert q(_rot(), T=0) == E_SHAPE
    assert q(_rot(), ldx=256) == E_SHAPE
    assert q(_rot(), ldx=513) == E_ALIGN
    assert q(_rot()) == E_UNSUP                       # no plan


def test_row_stride_limit():
    """Strides of 2^22 elements and more are refused before any launch (32-bit offsets inside a run of rows)."""
    L = paro.lib()
    big = 1 << 22
    assert L.paro_rotate_scale(ctypes.byref(_rot()), FAKE, big, FAKE, 512, 1, None) == E_UNSUP
    assert L.paro_rotate_scale(ctypes.byref(_rot()), FAKE, 512, FAKE, big, 1, None) == E_UNSUP
    w = _w(packed=FAKE)
    assert L.paro_w4a16_linear(ctypes.byref(w), FAKE, big, FAKE, 8192, 1, None, 0, None) == E_UNSUP
    assert L.paro_rotate_scale_quantize_mxfp4(ctypes.byref(_rot(plan=FAKE)), FAKE, big, 1, FAKE, FAKE, None) == E_UNSUP


def test_workspace_parts():
    """Exchange part <= total; a fused call (T <= 4, planned, repacked) needs no scratch, a separate rotation pass
    adds T * c_in * 2 bytes of it (rounded to 256).  The exchange part starts with the 256-byte header."""
    L = paro.lib()
    w = _w(c_in=2048, c_out=512, packed=FAKE)
    r = _rot(c_in=2048, plan=FAKE)
    for T in (1, 4, 5, 16, 300):
        tot, ex = L.paro_workspace_bytes(ctypes.byref(r), ctypes.byref(w), T), L.paro_workspace_exchange_bytes(
            ctypes.byref(r), ctypes.byref(w), T)
        assert ex <= tot and ex % 256 == 0
        assert ex >= 256
        xr = 0 if T <= 4 else (T * 2048 * 2 + 255) // 256 * 256
        bare = L.paro_workspace_bytes(None, ctypes.byref(w), T) - L.paro_workspace_exchange_bytes(None, ctypes.byref(w), T)
        assert tot - ex == xr + bare, (T, tot, ex)
        # the bare linear needs scratch only where the GEMM splits K (moderate token counts, few output tiles)
        assert (bare == 0) if T <= 16 else (bare % 256 == 0 and bare >= 2 * T * 512 * 4), (T, bare)
    r2 = _rot(c_in=2048)                                              # no plan: always a separate pass
    assert L.paro_workspace_bytes(ctypes.byref(r2), ctypes.byref(w), 1) - L.paro_workspace_exchange_bytes(
        ctypes.byref(r2), ctypes.byref(w), 1) == 4096
    assert L.paro_workspace_exchange_bytes(ctypes.byref(_rot(c_in=512)), ctypes.byref(w), 1) == 0     # mismatch: 0


def test_exchange_part_covers_the_partial_sums_of_every_shape():
    """Wherever a decode launch exchanges partial sums between blocks it stores K-parts x T x c_out fp32 words behind
    the 256-byte header; the size the library reports must cover them for every shape, also for one K-slice with a
    very wide output (no exchange at all: header only)."""
    L = paro.lib()
    for c_in in (512, 1024, 4096, 6144, 6656, 14336, 27648):
        for c_out in (16, 4096, 28672, 98304):
            for T in (1, 2, 4, 5, 16):
                w = _w(c_in=c_in, c_out=c_out, packed=FAKE)
                r = _rot(c_in=c_in, plan=FAKE)
                ks = c_in // 512
                fused = L.paro_workspace_bytes(ctypes.byref(r), ctypes.byref(w), T) == L.paro_workspace_exchange_bytes(
                    ctypes.byref(r), ctypes.byref(w), T)
                ex = L.paro_workspace_exchange_bytes(ctypes.byref(r), ctypes.byref(w), T)
                bare = L.paro_workspace_exchange_bytes(None, ctypes.byref(w), T)
                parts = 1 if ks <= 12 else (ks + 7) // 8                              # blocks along K of the bare kernel
                assert bare == (0 if parts == 1 else 256 + (parts * T * c_out * 4 + 255) // 256 * 256), (c_in, c_out, T, bare)
                # one token and at least 4 tiles per wave of the bare kernel's blocks (6 where a block has more than 8
                # waves): every wave transforms its own slice inside that block structure, which exchanges what the
                # bare kernel exchanges (plus the header)
                waves = -(-ks // parts)
                tiles = min(16, -(-(c_out // 16) // max(1, 256 // parts)))
                hosted_wide = T == 1 and tiles >= (4 if waves <= 8 else 6)
                if hosted_wide:
                    assert fused and ex == max(bare, 256), (c_in, c_out, T, ex, bare)
                elif T <= 4 and fused and ks > 1:
                    assert ex >= 256 + ks * T * c_out * 4, (c_in, c_out, T, ex)      # K-major kernel: one part per slice
                if ks == 1:
                    assert ex == 256, (c_in, c_out, T, ex)
                assert ex >= bare


def test_fused_or_two_launches_by_shape():
    """Up to 4 tokens a decode kernel hosts the rotation (no scratch part): at one token and from 4 tiles per wave
    the kernel whose waves each transform their own K-slice, otherwise the K-major kernel unless the partial
    sums its blocks would exchange (K-slices x T x c_out x 4 bytes) exceed 1.5 MB at one token or 0.75 MB at 2..4 -
    then the rotation runs as a pass of its own, which shows as a scratch part of T * c_in * 2 bytes."""
    L = paro.lib()

    def scratch(c_in, c_out, T):
        r, w = _rot(c_in=c_in, plan=FAKE), _w(c_in=c_in, c_out=c_out, packed=FAKE)
        return L.paro_workspace_bytes(ctypes.byref(r), ctypes.byref(w), T) - L.paro_workspace_exchange_bytes(
            ctypes.byref(r), ctypes.byref(w), T)

    assert scratch(4096, 6144, 1) == 0 and scratch(4096, 28672, 1) == 0 and scratch(14336, 4096, 1) == 0
    assert scratch(27648, 5120, 1) == 0                    # 54 slices x 5120 x 4 = 1.1 MB
    assert scratch(5120, 55296, 1) == 0                    # 14 tiles per wave: hosted by the waves of the bare kernel's blocks
    assert scratch(5120, 16384, 1) == 0                    # 10 x 16384 x 4 = 640 KB: K-major kernel
    assert scratch(5120, 14336, 2) == 2 * 5120 * 2         # 2 tokens, 10 x 2 x 14336 x 4 = 1.1 MB: two launches
    ex = lambda c_in, c_out, T: L.paro_workspace_exchange_bytes(
        ctypes.byref(_rot(c_in=c_in, plan=FAKE)), ctypes.byref(_w(c_in=c_in, c_out=c_out, packed=FAKE)), T)
    assert ex(4096, 28672, 1) == 256 and ex(5120, 55296, 1) == 256        # nothing exchanged between blocks
    assert ex(27648, 5120, 1) == 256 + 7 * 5120 * 4                       # 54 slices in 7 blocks of 8 waves
    assert ex(14336, 4096, 1) == 256 + 4 * 4096 * 4                       # 4 tiles per wave: hosted too (4 blocks of 7 waves per row)
    assert ex(6144, 12288, 1) == 256 + 12 * 12288 * 4                     # 12 waves, 3 tiles per wave: K-major kernel
    assert ex(4096, 6144, 1) == 256 + 8 * 6144 * 4                        # K-major kernel: one part per slice
    assert scratch(4096, 6144, 2) == 0 and scratch(4096, 4096, 3) == 0
    assert scratch(4096, 6144, 4) == 0                     # 8 x 4 x 6144 x 4 = 768 KiB: still hosted
    assert scratch(5120, 5120, 4) == 4 * 5120 * 2          # 10 x 4 x 5120 x 4 = 800 KiB
    assert scratch(4096, 28672, 2) == 2 * 4096 * 2


def test_mxfp4_linear_argument_errors():
    L = paro.lib()
    M = B._CMxfp4Weight
    ok = M(1024, 64, FAKE, FAKE, None, FAKE)
    lin = lambda w, xc=FAKE, xs=FAKE, T=1, Y=FAKE, ldy=64: L.paro_mxfp4_linear(ctypes.byref(w) if w else None, xc, xs, T, Y, ldy, None)
    assert lin(None) == E_NULL
    assert lin(ok, xc=None) == E_NULL and lin(ok, Y=None) == E_NULL
    assert lin(M(1024 + 128, 64, FAKE, FAKE, None, FAKE)) == E_SHAPE          # c_in not a multiple of 512
    assert lin(M(1024, 72, FAKE, FAKE, None, FAKE), ldy=72) == E_SHAPE        # c_out not a multiple of 16
    assert lin(ok, T=0) == E_SHAPE and lin(ok, ldy=32) == E_SHAPE
    assert lin(ok, xc=FAKE + 4) == E_ALIGN and lin(ok, xs=FAKE + 8) == E_ALIGN
    assert lin(M(1024, 64, FAKE, FAKE, None, None)) == E_UNSUP                # not repacked
    assert lin(M(32768, 64, FAKE, FAKE, None, FAKE)) == E_UNSUP               # more than 60 K-slices
    L.paro_mxfp4_packed_bytes.restype = ctypes.c_size_t
    assert L.paro_mxfp4_packed_bytes(ctypes.byref(ok)) == 1024 * 64 // 2 + 1024 * 64 // 32
    assert L.paro_mxfp4_packed_bytes(ctypes.byref(M(640, 64, FAKE, FAKE, None, None))) == 0
    assert L.paro_mxfp4_repack(ctypes.byref(M(1024, 64, None, FAKE, None, None)), FAKE, None) == E_NULL
    assert L.paro_mxfp4_repack(ctypes.byref(ok), FAKE + 16, None) == E_ALIGN
    q = lambda r, W=FAKE, ldw=1024, c_in=1024, c_out=64, c=FAKE, s=FAKE: L.paro_mxfp4_quantize_weight(
        ctypes.byref(r) if r else None, W, ldw, c_in, c_out, c, s, None)
    assert q(None, W=None) == E_NULL and q(None, c_in=1000) == E_SHAPE and q(None, ldw=512) == E_SHAPE
    assert q(_rot(c_in=512, plan=FAKE)) == E_SHAPE and q(_rot(c_in=1024)) == E_UNSUP
    L.paro_workspace_bytes_mxfp4.restype = ctypes.c_size_t
    assert L.paro_workspace_bytes_mxfp4(4096, 16) == 16 * 4096 // 2 + 16 * 4096 // 32
    assert L.paro_workspace_bytes_mxfp4(4096, 1) == 2048 + 256 and L.paro_workspace_bytes_mxfp4(640, 1) == 0
    full = lambda r, w, T=1, ws=FAKE, n=1 << 20: L.paro_rotated_linear_mxfp4(ctypes.byref(r), ctypes.byref(w), FAKE, 1024, FAKE, 64, T, ws, n, None)
    assert full(_rot(c_in=512, plan=FAKE), ok) == E_SHAPE
    assert full(_rot(c_in=1024), ok) == E_UNSUP
    assert full(_rot(c_in=1024, plan=FAKE), ok, n=100) == E_WS
    assert full(_rot(c_in=1024, plan=FAKE), ok, ws=FAKE + 64) == E_ALIGN


def test_fwht_argument_errors():
    L = paro.lib()
    assert L.paro_fwht(None, 64, FAKE, 64, 1, 64, None) == 1
    assert L.paro_fwht(FAKE, 64, FAKE, 64, 1, 48, None) == 2          # not a power of two
    assert L.paro_fwht(FAKE, 32, FAKE, 64, 1, 64, None) == 2          # ld < n
    assert L.paro_fwht(FAKE, 65536, FAKE, 65536, 1, 65536, None) == 5
    assert L.paro_fwht(FAKE + 2, 64, FAKE, 64, 1, 64, None) == 3
