"""ctypes front end of the scalar C oracle (oracle/tern_oracle.c).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it.  It shares no code with the GPU library and never calls it.

All arithmetic lives in the C file; this module only checks array types/shapes and chains the C
routines for the multi-layer encoder (conv -> threshold, layer by layer, on unpacked int8 tensors;
paper section 2, last paragraph: a module is a ternary convolution followed by batch-norm and the
ternary activation, and modules are chained).
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


class _Geom(C.Structure):
    _fields_ = [(k, C.c_int) for k in (
        "n", "c_in", "d", "h", "w", "c_out", "kd", "kh", "kw",
        "sd", "sh", "sw", "pd", "ph", "pw", "dd", "dh", "dw")]


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(_build.build())
        lib.oracle_max_threads.restype = C.c_int
        lib.oracle_set_threads.argtypes = [C.c_int]
        lib.oracle_set_threads.restype = None
        P = C.c_void_p
        lib.oracle_out_dims.argtypes = [C.POINTER(_Geom)] + [C.POINTER(C.c_int)] * 3
        lib.oracle_conv3d.argtypes = [C.POINTER(_Geom), P, P, P]
        lib.oracle_conv3d_points.argtypes = [C.POINTER(_Geom), P, P, P, C.c_int64, P]
        lib.oracle_threshold_i32.argtypes = [P, C.c_int, C.c_int, C.c_int64, P, P, P]
        lib.oracle_threshold_f32.argtypes = [P, C.c_int, C.c_int, C.c_int64, P, P, P]
        lib.oracle_pack.argtypes = [P, C.c_int, C.c_int, C.c_int64, P]
        lib.oracle_unpack.argtypes = [P, C.c_int, C.c_int, C.c_int64, P]
        _lib = lib
    return _lib


def _triple(v) -> Tuple[int, int, int]:
    if isinstance(v, (int, np.integer)):
        return (int(v),) * 3
    v = tuple(int(t) for t in v)
    if len(v) != 3:
        raise ValueError("expected an int or three ints")
    return v


@dataclass(frozen=True)
class ConvGeom:
    """Kernel extent, stride, zero padding and dilation per (depth, height, width) axis."""
    k: Tuple[int, int, int] = (3, 3, 3)
    stride: Tuple[int, int, int] = (1, 1, 1)
    pad: Tuple[int, int, int] = (1, 1, 1)
    dil: Tuple[int, int, int] = (1, 1, 1)

    @staticmethod
    def make(k=3, stride=1, pad=1, dil=1) -> "ConvGeom":
        return ConvGeom(_triple(k), _triple(stride), _triple(pad), _triple(dil))


def _cgeom(act_shape, c_out, g: ConvGeom) -> _Geom:
    n, c_in, d, h, w = (int(t) for t in act_shape)
    return _Geom(n, c_in, d, h, w, int(c_out), *g.k, *g.stride, *g.pad, *g.dil)


def _check(rc: int, what: str):
    if rc == -1:
        raise ValueError(f"{what}: invalid argument (extent, geometry or lo > hi)")
    if rc == -2:
        raise ValueError(f"{what}: value outside the ternary set / invalid 2-bit code")
    if rc != 0:
        raise RuntimeError(f"{what}: error {rc}")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _need(a, dtype, ndim=None, name="array") -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"{name} must be a C-contiguous numpy array of {np.dtype(dtype)}")
    if ndim is not None and a.ndim != ndim:
        raise ValueError(f"{name} must have {ndim} dimensions")
    return a


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def out_dims(act_shape, c_out: int, g: ConvGeom) -> Tuple[int, int, int]:
    cg = _cgeom(act_shape, c_out, g)
    od, oh, ow = C.c_int(), C.c_int(), C.c_int()
    _check(_load().oracle_out_dims(C.byref(cg), C.byref(od), C.byref(oh), C.byref(ow)), "out_dims")
    return od.value, oh.value, ow.value


def conv3d(act: np.ndarray, wgt: np.ndarray, g: ConvGeom) -> np.ndarray:
    """int32 accumulators [N][C_out][Do][Ho][Wo] of the ternary cross-correlation."""
    _need(act, np.int8, 5, "act")
    _need(wgt, np.int8, 5, "wgt")
    if wgt.shape[1] != act.shape[1] or tuple(wgt.shape[2:]) != tuple(g.k):
        raise ValueError("weight shape does not match C_in / kernel extent")
    cg = _cgeom(act.shape, wgt.shape[0], g)
    od, oh, ow = out_dims(act.shape, wgt.shape[0], g)
    acc = np.empty((act.shape[0], wgt.shape[0], od, oh, ow), dtype=np.int32)
    _check(_load().oracle_conv3d(C.byref(cg), _ptr(act), _ptr(wgt), _ptr(acc)), "conv3d")
    return acc


def conv3d_points(act: np.ndarray, wgt: np.ndarray, g: ConvGeom, pts: np.ndarray) -> np.ndarray:
    """Accumulators at output coordinates pts[i] = (n, c_out, z, y, x)."""
    _need(act, np.int8, 5, "act")
    _need(wgt, np.int8, 5, "wgt")
    pts = np.ascontiguousarray(pts, dtype=np.int32)
    if pts.ndim != 2 or pts.shape[1] != 5:
        raise ValueError("pts must be [P][5]")
    if wgt.shape[1] != act.shape[1] or tuple(wgt.shape[2:]) != tuple(g.k):
        raise ValueError("weight shape does not match C_in / kernel extent")
    cg = _cgeom(act.shape, wgt.shape[0], g)
    acc = np.empty((pts.shape[0],), dtype=np.int32)
    _check(_load().oracle_conv3d_points(C.byref(cg), _ptr(act), _ptr(wgt), _ptr(pts),
                                        pts.shape[0], _ptr(acc)), "conv3d_points")
    return acc


def threshold(v: np.ndarray, lo: np.ndarray, hi: np.ndarray) -> np.ndarray:
    """Ternary codes (int8) of an int32 or float32 [N][C][...] tensor: +1 if v > hi[c], -1 if
    v < lo[c], else 0 (Eq. 6 with the cut points given per channel)."""
    if not isinstance(v, np.ndarray) or v.ndim < 2 or not v.flags.c_contiguous:
        raise TypeError("v must be a C-contiguous numpy array [N][C][...]")
    n, c = v.shape[:2]
    spatial = int(np.prod(v.shape[2:], dtype=np.int64))
    code = np.empty(v.shape, dtype=np.int8)
    if v.dtype == np.int32:
        lo = _need(np.ascontiguousarray(lo), np.int32, 1, "lo")
        hi = _need(np.ascontiguousarray(hi), np.int32, 1, "hi")
        fn = _load().oracle_threshold_i32
    elif v.dtype == np.float32:
        lo = _need(np.ascontiguousarray(lo), np.float32, 1, "lo")
        hi = _need(np.ascontiguousarray(hi), np.float32, 1, "hi")
        fn = _load().oracle_threshold_f32
    else:
        raise TypeError("v must be int32 or float32")
    if lo.shape[0] != c or hi.shape[0] != c:
        raise ValueError("lo/hi must have one entry per channel")
    _check(fn(_ptr(v), n, c, spatial, _ptr(lo), _ptr(hi), _ptr(code)), "threshold")
    return code


def pack(x: np.ndarray) -> np.ndarray:
    """int8 ternary [N][C][...] -> uint32 [N][...][2][ceil(C/32)] (mask plane, sign plane)."""
    _need(x, np.int8, None, "x")
    if x.ndim < 2:
        raise ValueError("x must be [N][C][...]")
    n, c = x.shape[:2]
    spatial = int(np.prod(x.shape[2:], dtype=np.int64))
    words = (c + 31) // 32
    out = np.empty((n,) + tuple(x.shape[2:]) + (2, words), dtype=np.uint32)
    _check(_load().oracle_pack(_ptr(x), n, c, spatial, _ptr(out)), "pack")
    return out


def unpack(packed: np.ndarray, c: int) -> np.ndarray:
    """Inverse of pack(); rejects the unused fourth code point and stray bits above channel c."""
    _need(packed, np.uint32, None, "packed")
    words = (c + 31) // 32
    if packed.ndim < 3 or packed.shape[-2:] != (2, words):
        raise ValueError("packed must be [N][...][2][ceil(C/32)]")
    n = packed.shape[0]
    sp_shape = tuple(packed.shape[1:-2])
    spatial = int(np.prod(sp_shape, dtype=np.int64))
    x = np.empty((n, c) + sp_shape, dtype=np.int8)
    _check(_load().oracle_unpack(_ptr(packed), n, c, spatial, _ptr(x)), "unpack")
    return x


def fcn_forward(x: np.ndarray, in_lo: np.ndarray, in_hi: np.ndarray,
                layers: Sequence[dict], keep_acc: bool = False):
    """Chain of TernaryNet modules on unpacked tensors.

    x: float32 [N][C0][D][H][W] raw intensities, ternarised per channel at (in_lo, in_hi)
    (Eq. 6 uses -0.5 / +0.5).  layers: dicts with 'w' (int8 [C_out][C_in][kd][kh][kw]),
    'geom' (ConvGeom), 'lo', 'hi' (int32 [C_out]).  Returns the list of per-layer int8 codes
    (and, if keep_acc, the per-layer int32 accumulators).
    """
    cur = threshold(np.ascontiguousarray(x, dtype=np.float32), in_lo, in_hi)
    codes, accs = [], []
    for L in layers:
        acc = conv3d(cur, L["w"], L["geom"])
        cur = threshold(acc, L["lo"], L["hi"])
        codes.append(cur)
        if keep_acc:
            accs.append(acc)
    return (codes, accs) if keep_acc else codes
