"""ctypes binding of libparo.so.  Names follow include/paro.h one to one."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libparo.so")
_lib = None

PARO_OK = 0


class ParoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({paro_status_string(status)})")


class _CRotation(ctypes.Structure):
    _fields_ = [
        ("c_in", ctypes.c_int32), ("group", ctypes.c_int32), ("n_layers", ctypes.c_int32),
        ("pairs_per_layer", ctypes.c_int32),
        ("pairs", ctypes.c_void_p), ("theta", ctypes.c_void_p), ("ch_scale", ctypes.c_void_p),
        ("scale_order", ctypes.c_int32), ("plan", ctypes.c_void_p),
    ]


class _CW4Weight(ctypes.Structure):
    _fields_ = [
        ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32), ("group", ctypes.c_int32),
        ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("qzeros", ctypes.c_void_p),
        ("bias", ctypes.c_void_p), ("packed", ctypes.c_void_p),
    ]


class _CMxfp4Weight(ctypes.Structure):
    _fields_ = [
        ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32),
        ("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("packed", ctypes.c_void_p),
    ]


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Load libparo.so, building it first only if nothing has been built yet."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        rp, wp = ctypes.POINTER(_CRotation), ctypes.POINTER(_CW4Weight)
        L.paro_version.restype = ctypes.c_int
        L.paro_status_string.restype = ctypes.c_char_p
        L.paro_status_string.argtypes = [ctypes.c_int]
        L.paro_validate_pairs_host.argtypes = [vp, i32, i32, i32, i32]
        L.paro_select_pairs_host.argtypes = [vp, i32, i32, i32, vp, vp]
        L.paro_rotation_plan_bytes.restype = sz
        L.paro_rotation_plan_bytes.argtypes = [rp]
        L.paro_rotation_plan_build.argtypes = [rp, vp, vp]
        L.paro_w4_repack_bytes.restype = sz
        L.paro_w4_repack_bytes.argtypes = [wp]
        L.paro_w4_repack.argtypes = [wp, vp, vp]
        L.paro_workspace_bytes.restype = sz
        L.paro_workspace_bytes.argtypes = [rp, wp, i32]
        L.paro_workspace_exchange_bytes.restype = sz
        L.paro_workspace_error_offset.restype = sz
        L.paro_workspace_partials_offset.restype = sz
        L.paro_workspace_exchange_bytes.argtypes = [rp, wp, i32]
        L.paro_rotate_scale.argtypes = [rp, vp, i64, vp, i64, i32, vp]
        L.paro_w4a16_linear.argtypes = [wp, vp, i64, vp, i64, i32, vp, sz, vp]
        L.paro_rotated_linear.argtypes = [rp, wp, vp, i64, vp, i64, i32, vp, sz, vp]
        L.paro_rotated_linear_noalloc.argtypes = [rp, wp, vp, i64, vp, i64, i32, vp]
        L.paro_w4_unpack_codes.argtypes = [wp, vp, vp]
        L.paro_w4_unpack_zeros.argtypes = [wp, vp, vp]
        L.paro_w4_dequant.argtypes = [wp, vp, vp]
        L.paro_w4_quantize.argtypes = [rp, vp, i64, i32, i32, vp, vp, vp, vp]
        L.paro_rotate_scale_quantize_int4.argtypes = [rp, vp, i64, i32, vp, vp, vp, vp]
        L.paro_rotate_scale_quantize_mxfp4.argtypes = [rp, vp, i64, i32, vp, vp, vp]
        L.paro_workspace_bytes_multi.restype = sz
        L.paro_workspace_bytes_multi.argtypes = [i32, vp, vp, i32]
        L.paro_workspace_exchange_bytes_multi.restype = sz
        L.paro_workspace_exchange_bytes_multi.argtypes = [i32, vp, vp, i32]
        L.paro_rotated_linear_multi.argtypes = [i32, vp, vp, vp, i64, vp, vp, i32, vp, sz, vp]
        L.paro_fwht.argtypes = [vp, i64, vp, i64, i32, i32, vp]
        mp = ctypes.POINTER(_CMxfp4Weight)
        L.paro_mxfp4_quantize_weight.argtypes = [rp, vp, i64, i32, i32, vp, vp, vp]
        L.paro_mxfp4_packed_bytes.restype = sz
        L.paro_mxfp4_packed_bytes.argtypes = [mp]
        L.paro_mxfp4_repack.argtypes = [mp, vp, vp]
        L.paro_mxfp4_unpack.argtypes = [mp, vp, vp, vp]
        L.paro_mxfp4_linear.argtypes = [mp, vp, vp, i32, vp, i64, vp]
        L.paro_workspace_bytes_mxfp4.restype = sz
        L.paro_workspace_bytes_mxfp4.argtypes = [i32, i32]
        L.paro_rotated_linear_mxfp4.argtypes = [rp, mp, vp, i64, vp, i64, i32, vp, sz, vp]
        L.paro_diag_read_stream.argtypes = [vp, sz, vp, i32, vp]
        L.paro_diag_mfma_f16.argtypes = [vp, sz, i32, i32, i32, vp]
        L.paro_diag_mfma_f16_flops.argtypes = [i32, i32]
        L.paro_diag_mfma_f16_flops.restype = ctypes.c_double
        L.paro_diag_mfma_fp4.argtypes = [vp, sz, i32, i32, i32, vp]
        L.paro_diag_mfma_fp4.restype = ctypes.c_int
        L.paro_diag_mfma_fp4_flops.argtypes = [i32, i32]
        L.paro_diag_mfma_fp4_flops.restype = ctypes.c_double
        for name in ("paro_validate_pairs_host", "paro_select_pairs_host", "paro_rotation_plan_build", "paro_w4_repack", "paro_rotate_scale",
                     "paro_w4a16_linear", "paro_rotated_linear", "paro_rotated_linear_noalloc", "paro_w4_unpack_codes", "paro_w4_unpack_zeros",
                     "paro_w4_dequant", "paro_w4_quantize", "paro_rotated_linear_multi",
                     "paro_rotate_scale_quantize_int4", "paro_rotate_scale_quantize_mxfp4",
                     "paro_diag_read_stream", "paro_diag_mfma_f16", "paro_fwht", "paro_mxfp4_quantize_weight",
                     "paro_mxfp4_repack", "paro_mxfp4_unpack", "paro_mxfp4_linear", "paro_rotated_linear_mxfp4"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(st: int, where: str):
    if st != PARO_OK:
        raise ParoError(st, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def paro_version() -> int:
    return lib().paro_version()


def paro_status_string(status: int) -> str:
    return lib().paro_status_string(int(status)).decode()


def paro_validate_pairs_host(pairs: np.ndarray, group: int = 128) -> int:
    """Def. 1 on a host (numpy int16) pair table [G][K][P][2]; returns the status code."""
    p = np.ascontiguousarray(pairs, dtype=np.int16)
    G, K, P, two = p.shape
    assert two == 2
    return lib().paro_validate_pairs_host(p.ctypes.data, G, K, P, group)


def paro_fwht(X: torch.Tensor, Y: torch.Tensor | None = None) -> torch.Tensor:
    """Walsh-Hadamard transform of every row (Sylvester order, scaled by 1/sqrt(n))."""
    T, ldx = _rows(X)
    n = X.shape[1]
    if Y is None:
        Y = torch.empty((T, n), dtype=torch.float16, device=X.device)
    _, ldy = _rows(Y)
    _check(lib().paro_fwht(X.data_ptr(), ldx, Y.data_ptr(), ldy, T, n, _stream()), "paro_fwht")
    return Y


def paro_diag_read_stream(src: torch.Tensor, nbytes: int, blocks: int = 2048) -> None:
    """Pure-read ceiling probe over the first nbytes of src (a uint8 device tensor)."""
    assert src.dtype == torch.uint8 and src.numel() >= nbytes
    _check(lib().paro_diag_read_stream(src.data_ptr(), nbytes, None, blocks, _stream()), "paro_diag_read_stream")


def paro_diag_mfma_f16(out: torch.Tensor, blocks: int, iters: int, random_operands: bool) -> float:
    """Pure fp16 MFMA probe; returns the floating-point operations of the launch."""
    assert out.dtype == torch.float32 and out.numel() >= blocks * 256
    _check(lib().paro_diag_mfma_f16(out.data_ptr(), out.numel() * 4, blocks, iters, int(random_operands), _stream()),
           "paro_diag_mfma_f16")
    return lib().paro_diag_mfma_f16_flops(blocks, iters)


def paro_diag_mfma_fp4(out: torch.Tensor, blocks: int, iters: int, random_operands: bool) -> float:
    """Launch the FP4 MFMA issue probe; returns the floating-point operations of the launch."""
    _check(lib().paro_diag_mfma_fp4(out.data_ptr(), out.numel() * out.element_size(), blocks, iters, int(random_operands),
                                    _stream()), "paro_diag_mfma_fp4")
    return lib().paro_diag_mfma_fp4_flops(blocks, iters)


def paro_select_pairs_host(order: np.ndarray, group: int, n_rotations: int, pairs_per_rotation: int):
    """Algorithm A1 on a host permutation of the group's pairs; returns (pairs [K][N][2] int16, counts [K])."""
    o = np.ascontiguousarray(order, dtype=np.int32)
    assert o.shape == (group * (group - 1) // 2,)
    pairs = np.empty((n_rotations, pairs_per_rotation, 2), dtype=np.int16)
    counts = np.empty(n_rotations, dtype=np.int32)
    _check(lib().paro_select_pairs_host(o.ctypes.data, group, n_rotations, pairs_per_rotation, pairs.ctypes.data,
                                        counts.ctypes.data), "paro_select_pairs_host")
    return pairs, counts


class Rotation:
    """Device-side description of one linear's input transform (struct paro_rotation)."""

    def __init__(self, pairs, theta, ch_scale=None, scale_order: int = 0, group: int = 128, device="cuda"):
        self.pairs = torch.as_tensor(np.ascontiguousarray(pairs, dtype=np.int16)).to(device)
        self.theta = torch.as_tensor(np.ascontiguousarray(theta, dtype=np.float32)).to(device)
        G, K, P, _ = self.pairs.shape
        self.c_in = G * group
        self.ch_scale = None
        if ch_scale is not None:
            cs = np.ascontiguousarray(ch_scale)
            assert cs.dtype == np.float16 and cs.shape == (self.c_in,)
            self.ch_scale = torch.as_tensor(cs).to(device)
        self.plan = None
        self.c = _CRotation(self.c_in, group, K, P, _ptr(self.pairs), _ptr(self.theta), _ptr(self.ch_scale),
                            scale_order, None)

    def ref(self):
        return ctypes.byref(self.c)


class W4Weight:
    """Device-side INT4 group-quantised weight (struct paro_w4_weight)."""

    def __init__(self, qweight, scales, qzeros, bias=None, group: int = 128, device="cuda"):
        qw = np.ascontiguousarray(qweight, dtype=np.uint32)
        self.c_out, c8 = qw.shape
        self.c_in = c8 * 8
        sc = np.ascontiguousarray(scales)
        qz = np.ascontiguousarray(qzeros, dtype=np.uint32)
        assert sc.dtype == np.float16 and sc.shape == (self.c_in // group, self.c_out)
        assert qz.shape == (self.c_in // group, self.c_out // 8)
        self.qweight = torch.as_tensor(qw.view(np.int32)).to(device)
        self.scales = torch.as_tensor(sc).to(device)
        self.qzeros = torch.as_tensor(qz.view(np.int32)).to(device)
        self.bias = None if bias is None else torch.as_tensor(np.ascontiguousarray(bias, dtype=np.float16)).to(device)
        self.packed = None
        self.c = _CW4Weight(self.c_in, self.c_out, group, _ptr(self.qweight), _ptr(self.scales), _ptr(self.qzeros),
                            _ptr(self.bias), None)

    @classmethod
    def from_device(cls, qweight: torch.Tensor, scales: torch.Tensor, qzeros: torch.Tensor, bias=None, group: int = 128):
        """Wrap interchange-layout tensors that already live on the device (int32 / fp16 / int32)."""
        w = cls.__new__(cls)
        w.c_out, c8 = qweight.shape
        w.c_in = c8 * 8
        assert scales.shape == (w.c_in // group, w.c_out) and qzeros.shape == (w.c_in // group, w.c_out // 8)
        w.qweight, w.scales, w.qzeros, w.bias, w.packed = qweight, scales, qzeros, bias, None
        w.c = _CW4Weight(w.c_in, w.c_out, group, _ptr(qweight), _ptr(scales), _ptr(qzeros), _ptr(bias), None)
        return w

    def ref(self):
        return ctypes.byref(self.c)

    def drop_interchange(self):
        """Keep only the repacked blob (frees the interchange copies)."""
        assert self.packed is not None
        self.qweight = self.scales = self.qzeros = None
        self.c.qweight = self.c.scales = self.c.qzeros = None


class Workspace:
    """Zero-filled device workspace for the linear calls (see paro_workspace_bytes)."""

    def __init__(self, nbytes: int, device="cuda"):
        self.nbytes = int(nbytes)
        self.exchange_bytes = None          # set by shared(); None: unknown, taken to be present
        self.buf = torch.zeros(max(self.nbytes, 256), dtype=torch.uint8, device=device)

    def error_word(self) -> int:
        """The header's error word (synchronises): non-zero after an exchange between blocks timed out."""
        off = lib().paro_workspace_error_offset()
        if self.exchange_bytes is not None and self.exchange_bytes < off + 4:
            return 0                        # no exchange part: the buffer is scratch only
        return int(self.buf[off:off + 4].view(torch.int32).item()) if self.nbytes >= off + 4 else 0

    def partials_clean(self, exchange_bytes=None) -> bool:
        """True if the split-K partial sums of the exchange part are all zero again (synchronises)."""
        lo = lib().paro_workspace_partials_offset()
        hi = self.nbytes if exchange_bytes is None else exchange_bytes
        return hi <= lo or int(self.buf[lo:hi].max().item()) == 0

    @classmethod
    def shared(cls, calls, device="cuda"):
        """One workspace for calls of several shapes: calls = [(rot or None, weight, T), ...].  Sized as the
        largest exchange part plus the largest scratch part, so no call's scratch touches another's exchange part."""
        ex = sc = 0
        for rot, w, T in calls:
            total, e = paro_workspace_bytes(rot, w, T), paro_workspace_exchange_bytes(rot, w, T)
            ex, sc = max(ex, e), max(sc, total - e)
        ws = cls(ex + sc, device)
        ws.exchange_bytes = ex
        return ws


def paro_rotation_plan_build(rot: Rotation) -> None:
    n = lib().paro_rotation_plan_bytes(rot.ref())
    if n == 0:
        raise ParoError(5, "paro_rotation_plan_bytes")
    plan = torch.empty(n, dtype=torch.uint8, device=rot.pairs.device)
    _check(lib().paro_rotation_plan_build(rot.ref(), plan.data_ptr(), _stream()), "paro_rotation_plan_build")
    rot.plan = plan
    rot.c.plan = plan.data_ptr()


def paro_w4_repack(w: W4Weight) -> None:
    n = lib().paro_w4_repack_bytes(w.ref())
    if n == 0:
        raise ParoError(5, "paro_w4_repack_bytes")
    blob = torch.empty(n, dtype=torch.uint8, device=w.qweight.device)
    _check(lib().paro_w4_repack(w.ref(), blob.data_ptr(), _stream()), "paro_w4_repack")
    w.packed = blob
    w.c.packed = blob.data_ptr()


def paro_w4_quantize(rot: Rotation | None, W: torch.Tensor, group: int = 128) -> W4Weight:
    """Transform (Eq. 8, weight side) and RTN-quantise (Eq. 1) a dense fp16 weight [c_out][c_in]."""
    assert W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    c_out, c_in = W.shape
    qweight = torch.empty((c_out, c_in // 8), dtype=torch.int32, device=W.device)
    scales = torch.empty((c_in // group, c_out), dtype=torch.float16, device=W.device)
    qzeros = torch.empty((c_in // group, c_out // 8), dtype=torch.int32, device=W.device)
    _check(lib().paro_w4_quantize(rot.ref() if rot is not None else None, W.data_ptr(), W.stride(0), c_in, c_out,
                                  qweight.data_ptr(), scales.data_ptr(), qzeros.data_ptr(), _stream()),
           "paro_w4_quantize")
    return W4Weight.from_device(qweight, scales, qzeros, group=group)


def paro_workspace_bytes(rot: Rotation | None, w: W4Weight, T: int) -> int:
    return lib().paro_workspace_bytes(rot.ref() if rot is not None else None, w.ref(), T)


def paro_workspace_exchange_bytes(rot: Rotation | None, w: W4Weight, T: int) -> int:
    return lib().paro_workspace_exchange_bytes(rot.ref() if rot is not None else None, w.ref(), T)


def _rows(x: torch.Tensor):
    assert x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    return x.shape[0], x.stride(0)


def paro_rotate_scale(rot: Rotation, X: torch.Tensor, Xr: torch.Tensor | None = None) -> torch.Tensor:
    T, ldx = _rows(X)
    if Xr is None:
        Xr = torch.empty((T, rot.c_in), dtype=torch.float16, device=X.device)
    _, ldxr = _rows(Xr)
    _check(lib().paro_rotate_scale(rot.ref(), X.data_ptr(), ldx, Xr.data_ptr(), ldxr, T, _stream()), "paro_rotate_scale")
    return Xr


def paro_w4a16_linear(w: W4Weight, X: torch.Tensor, ws: Workspace | None = None, Y: torch.Tensor | None = None):
    T, ldx = _rows(X)
    if Y is None:
        Y = torch.empty((T, w.c_out), dtype=torch.float16, device=X.device)
    _, ldy = _rows(Y)
    _check(lib().paro_w4a16_linear(w.ref(), X.data_ptr(), ldx, Y.data_ptr(), ldy, T,
                                   ws.buf.data_ptr() if ws else None, ws.nbytes if ws else 0, _stream()),
           "paro_w4a16_linear")
    return Y


def paro_rotated_linear(rot: Rotation, w: W4Weight, X: torch.Tensor, ws: Workspace, Y: torch.Tensor | None = None):
    T, ldx = _rows(X)
    if Y is None:
        Y = torch.empty((T, w.c_out), dtype=torch.float16, device=X.device)
    _, ldy = _rows(Y)
    _check(lib().paro_rotated_linear(rot.ref(), w.ref(), X.data_ptr(), ldx, Y.data_ptr(), ldy, T,
                                     ws.buf.data_ptr(), ws.nbytes, _stream()), "paro_rotated_linear")
    return Y


def paro_rotated_linear_noalloc(rot: Rotation, w: W4Weight, X: torch.Tensor, Y: torch.Tensor):
    """paro_rotated_linear on the library's static exchange array: the caller passes inputs and outputs only."""
    T, ldx = _rows(X)
    _, ldy = _rows(Y)
    _check(lib().paro_rotated_linear_noalloc(rot.ref(), w.ref(), X.data_ptr(), ldx, Y.data_ptr(), ldy, T, _stream()),
           "paro_rotated_linear_noalloc")
    return Y


def paro_w4_unpack_codes(w: W4Weight) -> torch.Tensor:
    out = torch.empty((w.c_out, w.c_in), dtype=torch.uint8, device=(w.packed if w.qweight is None else w.qweight).device)
    _check(lib().paro_w4_unpack_codes(w.ref(), out.data_ptr(), _stream()), "paro_w4_unpack_codes")
    return out


def paro_w4_unpack_zeros(w: W4Weight) -> torch.Tensor:
    out = torch.empty((w.c_in // 128, w.c_out), dtype=torch.uint8, device=(w.packed if w.qweight is None else w.qweight).device)
    _check(lib().paro_w4_unpack_zeros(w.ref(), out.data_ptr(), _stream()), "paro_w4_unpack_zeros")
    return out


def paro_w4_dequant(w: W4Weight) -> torch.Tensor:
    out = torch.empty((w.c_out, w.c_in), dtype=torch.float16, device=(w.packed if w.qweight is None else w.qweight).device)
    _check(lib().paro_w4_dequant(w.ref(), out.data_ptr(), _stream()), "paro_w4_dequant")
    return out


def _ptr_array(objs):
    arr = (ctypes.c_void_p * len(objs))(*[ctypes.addressof(o.c) for o in objs])
    return arr


def paro_workspace_bytes_multi(rots, weights, T: int) -> int:
    assert len(rots) == len(weights)
    return lib().paro_workspace_bytes_multi(len(rots), _ptr_array(rots), _ptr_array(weights), T)


def paro_workspace_exchange_bytes_multi(rots, weights, T: int) -> int:
    assert len(rots) == len(weights)
    return lib().paro_workspace_exchange_bytes_multi(len(rots), _ptr_array(rots), _ptr_array(weights), T)


def paro_rotated_linear_multi(rots, weights, x: torch.Tensor, ws: Workspace, ys=None):
    """Several linears on the same x, each with its own transform (q / k / v, gate / up); returns the list of outputs."""
    T, ldx = _rows(x)
    n = len(rots)
    assert n == len(weights)
    if ys is None:
        ys = [torch.empty((T, w.c_out), dtype=torch.float16, device=x.device) for w in weights]
    y_ptrs = (ctypes.c_void_p * n)(*[y.data_ptr() for y in ys])
    ldys = (ctypes.c_int64 * n)(*[_rows(y)[1] for y in ys])
    _check(lib().paro_rotated_linear_multi(n, _ptr_array(rots), _ptr_array(weights), x.data_ptr(), ldx, y_ptrs, ldys, T,
                                           ws.buf.data_ptr(), ws.nbytes, _stream()), "paro_rotated_linear_multi")
    return ys


def paro_rotate_scale_quantize_int4(rot: Rotation, X: torch.Tensor):
    """Transform, then INT4-quantise per (token, group): returns (codes int32 [T][C/8], scales fp16 [T][G], zeros uint8 [T][G])."""
    T, ldx = _rows(X)
    C, G = rot.c_in, rot.c_in // 128
    codes = torch.empty((T, C // 8), dtype=torch.int32, device=X.device)
    scales = torch.empty((T, G), dtype=torch.float16, device=X.device)
    zeros = torch.empty((T, G), dtype=torch.uint8, device=X.device)
    _check(lib().paro_rotate_scale_quantize_int4(rot.ref(), X.data_ptr(), ldx, T, codes.data_ptr(), scales.data_ptr(),
                                                 zeros.data_ptr(), _stream()), "paro_rotate_scale_quantize_int4")
    return codes, scales, zeros


def paro_rotate_scale_quantize_mxfp4(rot: Rotation, X: torch.Tensor):
    """Transform, then MXFP4-quantise per (token, 32 channels): returns (codes int32 [T][C/8], scales uint8 [T][C/32])."""
    T, ldx = _rows(X)
    C = rot.c_in
    codes = torch.empty((T, C // 8), dtype=torch.int32, device=X.device)
    scales = torch.empty((T, C // 32), dtype=torch.uint8, device=X.device)
    _check(lib().paro_rotate_scale_quantize_mxfp4(rot.ref(), X.data_ptr(), ldx, T, codes.data_ptr(), scales.data_ptr(),
                                                  _stream()), "paro_rotate_scale_quantize_mxfp4")
    return codes, scales


class Mxfp4Weight:
    """Device-side MXFP4 weight (struct paro_mxfp4_weight): codes int32 [c_out][c_in/8], scales uint8 [c_out][c_in/32]."""

    def __init__(self, codes: torch.Tensor, scales: torch.Tensor, bias: torch.Tensor | None = None):
        self.c_out, c8 = codes.shape
        self.c_in = c8 * 8
        assert codes.dtype == torch.int32 and scales.dtype == torch.uint8 and scales.shape == (self.c_out, self.c_in // 32)
        self.codes, self.scales, self.bias, self.packed = codes, scales, bias, None
        self.c = _CMxfp4Weight(self.c_in, self.c_out, _ptr(codes), _ptr(scales), _ptr(bias), None)

    @classmethod
    def from_host(cls, codes_bytes: np.ndarray, scales: np.ndarray, bias=None, device="cuda"):
        """codes_bytes: uint8 [c_out][c_in] (one E2M1 code per byte), scales: uint8 [c_out][c_in/32]."""
        cb = np.ascontiguousarray(codes_bytes, dtype=np.uint8)
        n, c = cb.shape
        words = np.zeros((n, c // 8), dtype=np.uint32)
        for k in range(8):
            words |= cb[:, k::8].astype(np.uint32) << np.uint32(4 * k)
        b = None if bias is None else torch.as_tensor(np.ascontiguousarray(bias, dtype=np.float16)).to(device)
        return cls(torch.as_tensor(words.view(np.int32)).to(device),
                   torch.as_tensor(np.ascontiguousarray(scales, dtype=np.uint8)).to(device), b)

    def ref(self):
        return ctypes.byref(self.c)


def paro_mxfp4_quantize_weight(rot: Rotation | None, W: torch.Tensor, bias: torch.Tensor | None = None) -> Mxfp4Weight:
    """Q(T W) of App. A.3: weight-side transform, then MXFP4 per 32 channels, of a dense fp16 weight [c_out][c_in]."""
    assert W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    c_out, c_in = W.shape
    codes = torch.empty((c_out, c_in // 8), dtype=torch.int32, device=W.device)
    scales = torch.empty((c_out, c_in // 32), dtype=torch.uint8, device=W.device)
    _check(lib().paro_mxfp4_quantize_weight(rot.ref() if rot is not None else None, W.data_ptr(), W.stride(0), c_in, c_out,
                                            codes.data_ptr(), scales.data_ptr(), _stream()), "paro_mxfp4_quantize_weight")
    return Mxfp4Weight(codes, scales, bias)


def paro_mxfp4_repack(w: Mxfp4Weight) -> None:
    n = lib().paro_mxfp4_packed_bytes(w.ref())
    if n == 0:
        raise ParoError(5, "paro_mxfp4_packed_bytes")
    blob = torch.empty(n, dtype=torch.uint8, device=w.codes.device)
    _check(lib().paro_mxfp4_repack(w.ref(), blob.data_ptr(), _stream()), "paro_mxfp4_repack")
    w.packed = blob
    w.c.packed = blob.data_ptr()


def paro_mxfp4_unpack(w: Mxfp4Weight):
    """Test hook: (codes uint8 [c_out][c_in], scales uint8 [c_out][c_in/32]) from the repacked blob if present."""
    dev = w.packed.device if w.packed is not None else w.codes.device
    codes = torch.empty((w.c_out, w.c_in), dtype=torch.uint8, device=dev)
    scales = torch.empty((w.c_out, w.c_in // 32), dtype=torch.uint8, device=dev)
    _check(lib().paro_mxfp4_unpack(w.ref(), codes.data_ptr(), scales.data_ptr(), _stream()), "paro_mxfp4_unpack")
    return codes, scales


def paro_mxfp4_linear(w: Mxfp4Weight, x_codes: torch.Tensor, x_scales: torch.Tensor, Y: torch.Tensor | None = None):
    """Y' = Q(X T^-1) . Q(T W) + b on MXFP4 operands (App. A.3)."""
    T = x_codes.shape[0]
    assert x_codes.dtype == torch.int32 and x_codes.shape == (T, w.c_in // 8) and x_codes.is_contiguous()
    assert x_scales.dtype == torch.uint8 and x_scales.shape == (T, w.c_in // 32) and x_scales.is_contiguous()
    if Y is None:
        Y = torch.empty((T, w.c_out), dtype=torch.float16, device=x_codes.device)
    _, ldy = _rows(Y)
    _check(lib().paro_mxfp4_linear(w.ref(), x_codes.data_ptr(), x_scales.data_ptr(), T, Y.data_ptr(), ldy, _stream()),
           "paro_mxfp4_linear")
    return Y


def paro_workspace_bytes_mxfp4(c_in: int, T: int) -> int:
    return lib().paro_workspace_bytes_mxfp4(c_in, T)


def paro_rotated_linear_mxfp4(rot: Rotation, w: Mxfp4Weight, X: torch.Tensor, ws: torch.Tensor, Y: torch.Tensor | None = None):
    """Transform + MXFP4-quantise the activations into `ws` (uint8 tensor), then the MXFP4 x MXFP4 linear."""
    T, ldx = _rows(X)
    if Y is None:
        Y = torch.empty((T, w.c_out), dtype=torch.float16, device=X.device)
    _, ldy = _rows(Y)
    _check(lib().paro_rotated_linear_mxfp4(rot.ref(), w.ref(), X.data_ptr(), ldx, Y.data_ptr(), ldy, T, ws.data_ptr(),
                                           ws.numel(), _stream()), "paro_rotated_linear_mxfp4")
    return Y
