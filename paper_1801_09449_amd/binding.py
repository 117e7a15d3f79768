"""ctypes binding of libtern.so (the C ABI of include/tern.h) for torch device tensors.

Each function mirrors the C entry point of the same name: it checks tensor dtype / device /
contiguity, allocates the output tensor when the caller does not pass one, and forwards raw device
pointers plus the current torch stream.  No arithmetic happens here.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libtern.so"
_lib = None


class TernError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = lib().tern_status_string(status).decode() if _lib is not None else str(status)
        if status == -5:
            msg += f" (hipError_t {lib().tern_last_hip_error()})"
        super().__init__(f"{what}: {msg}")


class Dims(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n", "c", "d", "h", "w")]


class Geom(C.Structure):
    _fields_ = [("k", C.c_int32 * 3), ("stride", C.c_int32 * 3), ("pad", C.c_int32 * 3),
                ("dil", C.c_int32 * 3)]


class Layer(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32), ("g", Geom),
                ("w_bank", C.c_void_p), ("thr_lo", C.c_void_p), ("thr_hi", C.c_void_p)]


class Source(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("dims", Dims), ("up", C.c_int32 * 3),
                ("first", C.c_int32 * 3)]


class Module(C.Structure):
    _fields_ = [("c_out", C.c_int32), ("g", Geom), ("w_bank", C.c_void_p), ("thr_lo", C.c_void_p),
                ("thr_hi", C.c_void_p), ("skip_from", C.c_int32), ("up", C.c_int32 * 3),
                ("pool", C.c_int32 * 3)]


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def lib():
    """Load libtern.so (built in-tree by paper_1801_09449_amd/build.py).  Raises if missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_1801_09449_amd.build` "
            "(there is no fallback implementation)")
    L = C.CDLL(path)
    P, I, S = C.c_void_p, C.c_int32, C.c_size_t
    L.tern_words.argtypes = [I]; L.tern_words.restype = I
    L.tern_packed_bytes.argtypes = [Dims]; L.tern_packed_bytes.restype = S
    L.tern_filter_bank_bytes.argtypes = [I] * 5; L.tern_filter_bank_bytes.restype = S
    L.tern_conv_out_dims.argtypes = [Dims, I, Geom, C.POINTER(Dims)]; L.tern_conv_out_dims.restype = C.c_int
    L.tern_last_hip_error.argtypes = []; L.tern_last_hip_error.restype = C.c_int
    L.tern_status_string.argtypes = [C.c_int]; L.tern_status_string.restype = C.c_char_p
    L.tern_pack.argtypes = [P, Dims, P, P]; L.tern_pack.restype = C.c_int
    L.tern_pack_filters.argtypes = [P, I, I, I, I, I, P, P]; L.tern_pack_filters.restype = C.c_int
    L.tern_conv3d.argtypes = [P, Dims, P, I, Geom, P, P, P, P, P]; L.tern_conv3d.restype = C.c_int
    L.tern_conv3d_digits.argtypes = [P, Dims, P, I, Geom, P, P, P, P, P]; L.tern_conv3d_digits.restype = C.c_int
    L.tern_binary_bank_bytes.argtypes = [I] * 5; L.tern_binary_bank_bytes.restype = S
    L.tern_pack_filters_binary.argtypes = [P, I, I, I, I, I, P, P]; L.tern_pack_filters_binary.restype = C.c_int
    L.tern_conv3d_binary.argtypes = [P, Dims, P, I, Geom, P, P, P, P, P]; L.tern_conv3d_binary.restype = C.c_int
    L.tern_conv3d_mfma.argtypes = [P, Dims, P, I, I, Geom, P, P, P, P, P]; L.tern_conv3d_mfma.restype = C.c_int
    L.tern_matrix_bank_bytes.argtypes = [I] * 6; L.tern_matrix_bank_bytes.restype = S
    L.tern_conv3d_mfma_digits.argtypes = [P, Dims, P, I, Geom, P, P, P, P, P]; L.tern_conv3d_mfma_digits.restype = C.c_int
    L.tern_expand_filters.argtypes = [P, I, I, I, I, I, I, P, P]; L.tern_expand_filters.restype = C.c_int
    L.tern_pool_digits.argtypes = [P, Dims, C.POINTER(C.c_int32), P, P]; L.tern_pool_digits.restype = C.c_int
    L.tern_digits_weights.argtypes = [P, I, I, C.c_int64, P]; L.tern_digits_weights.restype = C.c_int
    L.tern_threshold_pack.argtypes = [P, C.c_int, Dims, P, P, P, P]; L.tern_threshold_pack.restype = C.c_int
    L.tern_fcn_workspace_bytes.argtypes = [Dims, C.POINTER(Layer), I]; L.tern_fcn_workspace_bytes.restype = S
    L.tern_fcn_forward.argtypes = [P, Dims, P, P, C.POINTER(Layer), I, P, S, P, C.POINTER(Dims),
                                   C.POINTER(C.c_void_p), P]
    L.tern_fcn_forward.restype = C.c_int
    L.tern_static_scratch_bytes.argtypes = []; L.tern_static_scratch_bytes.restype = S
    L.tern_fcn_forward_static.argtypes = [P, Dims, P, P, C.POINTER(Layer), I, P, C.POINTER(Dims),
                                          C.POINTER(C.c_void_p), P]
    L.tern_fcn_forward_static.restype = C.c_int
    L.tern_ternarize_filters.argtypes = [P, I, C.c_int64, P, P]; L.tern_ternarize_filters.restype = C.c_int
    L.tern_ternarize_filters_sparse.argtypes = [P, I, C.c_int64, C.c_int64, P, P]
    L.tern_ternarize_filters_sparse.restype = C.c_int
    L.tern_fold_thresholds.argtypes = [P, P, I, I, P, P, P]; L.tern_fold_thresholds.restype = C.c_int
    L.tern_fold_batchnorm.argtypes = [P, P, P, P, P, C.c_double, I, I, P, P, P]
    L.tern_fold_batchnorm.restype = C.c_int
    L.tern_concat.argtypes = [C.POINTER(Source), I, Dims, P, P]; L.tern_concat.restype = C.c_int
    L.tern_conv3d_real.argtypes = [P, Dims, P, P, I, Geom, P, P]; L.tern_conv3d_real.restype = C.c_int
    L.tern_net_workspace_bytes.argtypes = [Dims, C.POINTER(Module), I]; L.tern_net_workspace_bytes.restype = S
    L.tern_net_forward.argtypes = [P, Dims, P, P, C.POINTER(Module), I, P, P, I, Geom, P, S, P, C.POINTER(Dims),
                                   C.POINTER(C.c_void_p), C.POINTER(Dims), P]
    L.tern_net_forward.restype = C.c_int
    L.tern_count_codes.argtypes = [P, Dims, P, P, P]; L.tern_count_codes.restype = C.c_int
    L.tern_fold_avgpool.argtypes = [P, I, I, I, I, I, C.POINTER(C.c_int32), P]
    L.tern_fold_avgpool.restype = C.c_int
    L.tern_set_option.argtypes = [C.c_int, C.c_int]; L.tern_set_option.restype = C.c_int
    L.tern_probe_valu.argtypes = [I, I, I, I, P, P]; L.tern_probe_valu.restype = C.c_int
    L.tern_last_launch.argtypes = [C.POINTER(C.c_int32)]; L.tern_last_launch.restype = C.c_int
    _lib = L
    return L


# ---- helpers -----------------------------------------------------------------------------------
def _t3(v) -> Tuple[int, int, int]:
    if isinstance(v, int):
        return (v, v, v)
    v = tuple(int(x) for x in v)
    if len(v) != 3:
        raise ValueError("expected an int or three ints")
    return v


def _geom(k, stride, pad, dil) -> Geom:
    g = Geom()
    for name, val in (("k", k), ("stride", stride), ("pad", pad), ("dil", dil)):
        t = _t3(val)
        for i in range(3):
            getattr(g, name)[i] = t[i]
    return g


def _dims(shape) -> Dims:
    n, c, d, h, w = (int(x) for x in shape)
    return Dims(n, c, d, h, w)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch tensor")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (there is no CPU path)")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _stream(t: torch.Tensor) -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise TernError(rc, what)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


# torch has no uint32 arithmetic worth the name; packed words are carried as int32 tensors (same
# bits) and viewed as uint32 by whoever inspects them on the host.
PACKED_DTYPE = torch.int32


def tern_words(c: int) -> int:
    return int(lib().tern_words(int(c)))


def tern_packed_bytes(shape) -> int:
    return int(lib().tern_packed_bytes(_dims(shape)))


def tern_filter_bank_bytes(c_out: int, c_in: int, k) -> int:
    kd, kh, kw = _t3(k)
    return int(lib().tern_filter_bank_bytes(int(c_out), int(c_in), kd, kh, kw))


def tern_conv_out_dims(in_shape, c_out: int, k=3, stride=1, pad=1, dil=1) -> Tuple[int, ...]:
    o = Dims()
    _check(lib().tern_conv_out_dims(_dims(in_shape), int(c_out), _geom(k, stride, pad, dil), C.byref(o)),
           "tern_conv_out_dims")
    return (o.n, o.c, o.d, o.h, o.w)


def _empty_packed(shape, device) -> torch.Tensor:
    n, c, d, h, w = (int(x) for x in shape)
    return torch.empty((n, d, h, w, 2, tern_words(c)), dtype=PACKED_DTYPE, device=device)


# ---- entry points ------------------------------------------------------------------------------
def tern_pack(src: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int8 ternary [N][C][D][H][W] -> packed planes [N][D][H][W][2][ceil(C/32)] (int32 bits)."""
    _dev(src, torch.int8, "src")
    if src.dim() != 5:
        raise ValueError("src must be [N][C][D][H][W]")
    if out is None:
        out = _empty_packed(src.shape, src.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != tern_packed_bytes(src.shape):
        raise ValueError("out has the wrong size")
    _check(lib().tern_pack(_ptr(src), _dims(src.shape), _ptr(out), _stream(src)), "tern_pack")
    return out


def tern_pack_filters(w: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int8 ternary [C_out][C_in][kd][kh][kw] -> filter bank (flat int32 tensor)."""
    _dev(w, torch.int8, "w")
    if w.dim() != 5:
        raise ValueError("w must be [C_out][C_in][kd][kh][kw]")
    co, ci, kd, kh, kw = (int(x) for x in w.shape)
    nbytes = tern_filter_bank_bytes(co, ci, (kd, kh, kw))
    if nbytes == 0:
        raise TernError(-2, "tern_pack_filters")
    if out is None:
        out = torch.empty((nbytes // 4,), dtype=PACKED_DTYPE, device=w.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != nbytes:
        raise ValueError("out has the wrong size")
    _check(lib().tern_pack_filters(_ptr(w), co, ci, kd, kh, kw, _ptr(out), _stream(w)), "tern_pack_filters")
    return out


def tern_binary_bank_bytes(c_out: int, c_in: int, k) -> int:
    kd, kh, kw = _t3(k)
    return int(lib().tern_binary_bank_bytes(int(c_out), int(c_in), kd, kh, kw))


def tern_pack_filters_binary(w: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int8 weights in {-1, +1} [C_out][C_in][kd][kh][kw] -> binary filter bank (flat int32 tensor)."""
    _dev(w, torch.int8, "w")
    if w.dim() != 5:
        raise ValueError("w must be [C_out][C_in][kd][kh][kw]")
    co, ci, kd, kh, kw = (int(x) for x in w.shape)
    nbytes = tern_binary_bank_bytes(co, ci, (kd, kh, kw))
    if nbytes == 0:
        raise TernError(-2, "tern_pack_filters_binary")
    if out is None:
        out = torch.empty((nbytes // 4,), dtype=PACKED_DTYPE, device=w.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != nbytes:
        raise ValueError("out has the wrong size")
    _check(lib().tern_pack_filters_binary(_ptr(w), co, ci, kd, kh, kw, _ptr(out), _stream(w)),
           "tern_pack_filters_binary")
    return out


def tern_conv3d_binary(in_packed: torch.Tensor, c_in: int, w_bank: torch.Tensor, c_out: int,
                       k=3, stride=1, pad=1, dil=1, thr_lo: Optional[torch.Tensor] = None,
                       thr_hi: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """tern_conv3d with the binary filter bank of tern_pack_filters_binary (Eq. 8)."""
    return tern_conv3d(in_packed, c_in, w_bank, c_out, k, stride, pad, dil, thr_lo, thr_hi, out, binary=True)


MATRIX_KINDS = {"i8": 0, "f4": 1}


def tern_matrix_bank_bytes(c_out: int, c_in: int, k, kind: str = "i8") -> int:
    kd, kh, kw = _t3(k)
    return int(lib().tern_matrix_bank_bytes(int(c_out), int(c_in), kd, kh, kw, MATRIX_KINDS[kind]))


def tern_expand_filters(w: torch.Tensor, kind: str = "i8", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int8 ternary [C_out][C_in][kd][kh][kw] -> filter bank of the matrix-core route (flat int32
    tensor); kind "i8" (a byte per code) or "f4" (four bits per code)."""
    _dev(w, torch.int8, "w")
    if w.dim() != 5:
        raise ValueError("w must be [C_out][C_in][kd][kh][kw]")
    co, ci, kd, kh, kw = (int(x) for x in w.shape)
    nbytes = tern_matrix_bank_bytes(co, ci, (kd, kh, kw), kind)
    if nbytes == 0:
        raise TernError(-2, "tern_expand_filters")
    if out is None:
        out = torch.empty((nbytes // 4,), dtype=PACKED_DTYPE, device=w.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != nbytes:
        raise ValueError("out has the wrong size")
    _check(lib().tern_expand_filters(_ptr(w), co, ci, kd, kh, kw, MATRIX_KINDS[kind], _ptr(out), _stream(w)),
           "tern_expand_filters")
    return out


def tern_conv3d(in_packed: torch.Tensor, c_in: int, w_bank: torch.Tensor, c_out: int,
                k=3, stride=1, pad=1, dil=1,
                thr_lo: Optional[torch.Tensor] = None, thr_hi: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None, digits: bool = False,
                mfma=False, binary: bool = False) -> torch.Tensor:
    """Ternary convolution.  Without cut points: int32 accumulators [N][C_out][Do][Ho][Wo].
    With thr_lo / thr_hi (int32 [C_out]): fused activation + re-pack, packed output.
    digits=True: in_packed is the two-digit tensor of tern_pool_digits (c_in = its channel count,
    a multiple of 64) and w_bank the bank of tern_digits_weights' output (tern_conv3d_digits).
    mfma="i8" / "f4" (True = "i8"): w_bank is the bank of tern_expand_filters for that kind
    (tern_conv3d_mfma)."""
    kind = "i8" if mfma is True else mfma
    if binary and (digits or mfma):
        raise ValueError("binary filters go with neither digits nor mfma")
    if binary:
        entry = lib().tern_conv3d_binary
    elif digits and mfma:
        if kind != "f4":
            raise ValueError("two-digit inputs go through the 4-bit kind")
        entry = lib().tern_conv3d_mfma_digits
    elif mfma:
        def entry(a, d, b, *rest):
            return lib().tern_conv3d_mfma(a, d, b, MATRIX_KINDS[kind], *rest)
    else:
        entry = lib().tern_conv3d_digits if digits else lib().tern_conv3d
    _dev(in_packed, PACKED_DTYPE, "in_packed")
    _dev(w_bank, PACKED_DTYPE, "w_bank")
    if in_packed.dim() != 6 or in_packed.shape[4] != 2 or in_packed.shape[5] != tern_words(c_in):
        raise ValueError("in_packed must be [N][D][H][W][2][ceil(C_in/32)]")
    n, d, h, w = (int(x) for x in in_packed.shape[:4])
    in_dims = Dims(n, int(c_in), d, h, w)
    g = _geom(k, stride, pad, dil)
    kk = (g.k[0], g.k[1], g.k[2])
    if binary:
        need = tern_binary_bank_bytes(c_out, c_in, kk)
    elif digits and mfma:      # the bank of the undoubled weights: half the digit tensor's channels
        need = tern_matrix_bank_bytes(c_out, c_in // 2, kk, kind)
    else:
        need = tern_matrix_bank_bytes(c_out, c_in, kk, kind) if mfma else tern_filter_bank_bytes(c_out, c_in, kk)
    if w_bank.numel() * 4 != need:
        raise ValueError("w_bank size does not match (c_out, c_in, k)")
    o = Dims()
    _check(lib().tern_conv_out_dims(in_dims, int(c_out), g, C.byref(o)), "tern_conv3d")
    fused = thr_lo is not None or thr_hi is not None
    if fused:
        if thr_lo is None or thr_hi is None:
            raise ValueError("thr_lo and thr_hi must be given together")
        _dev(thr_lo, torch.int32, "thr_lo"); _dev(thr_hi, torch.int32, "thr_hi")
        if thr_lo.numel() != c_out or thr_hi.numel() != c_out:
            raise ValueError("cut points must have c_out entries")
        if out is None:
            out = _empty_packed((o.n, o.c, o.d, o.h, o.w), in_packed.device)
        _dev(out, PACKED_DTYPE, "out")
        if out.numel() * 4 != tern_packed_bytes((o.n, o.c, o.d, o.h, o.w)):
            raise ValueError("out has the wrong size")
        rc = entry(_ptr(in_packed), in_dims, _ptr(w_bank), int(c_out), g, _ptr(thr_lo),
                   _ptr(thr_hi), None, _ptr(out), _stream(in_packed))
    else:
        if out is None:
            out = torch.empty((o.n, o.c, o.d, o.h, o.w), dtype=torch.int32, device=in_packed.device)
        _dev(out, torch.int32, "out")
        if tuple(out.shape) != (o.n, o.c, o.d, o.h, o.w):
            raise ValueError("out has the wrong shape")
        rc = entry(_ptr(in_packed), in_dims, _ptr(w_bank), int(c_out), g, None, None,
                   _ptr(out), None, _stream(in_packed))
    _check(rc, "tern_conv3d")
    return out


def tern_pool_digits(in_packed: torch.Tensor, c: int, window, out: Optional[torch.Tensor] = None):
    """Sums over non-overlapping windows (at most 4 voxels) of a packed tensor, as two balanced-
    ternary digits: returns (packed [N][D'][H'][W'][2][2*words(c)], channel count 64*words(c))."""
    _dev(in_packed, PACKED_DTYPE, "in_packed")
    if in_packed.dim() != 6 or in_packed.shape[4] != 2 or in_packed.shape[5] != tern_words(c):
        raise ValueError("in_packed must be [N][D][H][W][2][ceil(C/32)]")
    win = _t3(window)
    n, d, h, w = (int(x) for x in in_packed.shape[:4])
    c2 = 64 * tern_words(c)
    if min(win) < 1:
        raise ValueError("window entries must be positive")
    shape = (n, c2, d // win[0], h // win[1], w // win[2])
    if out is None:
        out = _empty_packed(shape, in_packed.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != tern_packed_bytes(shape):
        raise ValueError("out has the wrong size")
    arr = (C.c_int32 * 3)(*win)
    _check(lib().tern_pool_digits(_ptr(in_packed), Dims(n, int(c), d, h, w), arr, _ptr(out), _stream(in_packed)),
           "tern_pool_digits")
    return out, c2


def tern_digits_weights(w):
    """int8 host weights [C_out][C_in][...] -> [C_out][64*words(C_in)][...] for tern_conv3d(digits=True)."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.int8)
    if w.ndim < 2:
        raise ValueError("w must be [C_out][C_in][...]")
    c_out, c_in = w.shape[:2]
    taps = int(w.size // (c_out * c_in))
    out = np.empty((c_out, 64 * tern_words(c_in)) + w.shape[2:], dtype=np.int8)
    _check(lib().tern_digits_weights(_np_ptr(w), c_out, c_in, taps, _np_ptr(out)), "tern_digits_weights")
    return out


def tern_threshold_pack(src: torch.Tensor, thr_lo: torch.Tensor, thr_hi: torch.Tensor,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """int32 or float32 [N][C][D][H][W] -> packed ternary codes (+1 if v > hi[c], -1 if v < lo[c])."""
    if not isinstance(src, torch.Tensor) or src.dtype not in (torch.int32, torch.float32):
        raise TypeError("src must be an int32 or float32 torch tensor")
    _dev(src, src.dtype, "src")
    if src.dim() != 5:
        raise ValueError("src must be [N][C][D][H][W]")
    _dev(thr_lo, src.dtype, "thr_lo"); _dev(thr_hi, src.dtype, "thr_hi")
    if thr_lo.numel() != src.shape[1] or thr_hi.numel() != src.shape[1]:
        raise ValueError("cut points must have C entries")
    if out is None:
        out = _empty_packed(src.shape, src.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != tern_packed_bytes(src.shape):
        raise ValueError("out has the wrong size")
    t = 1 if src.dtype == torch.int32 else 2
    _check(lib().tern_threshold_pack(_ptr(src), t, _dims(src.shape), _ptr(thr_lo), _ptr(thr_hi),
                                     _ptr(out), _stream(src)), "tern_threshold_pack")
    return out


@dataclass
class FcnLayer:
    """One module of the chain: filter bank + geometry + integer cut points (device tensors)."""
    c_in: int
    c_out: int
    w_bank: torch.Tensor
    thr_lo: torch.Tensor
    thr_hi: torch.Tensor
    k: Tuple[int, int, int] = (3, 3, 3)
    stride: Tuple[int, int, int] = (1, 1, 1)
    pad: Tuple[int, int, int] = (1, 1, 1)
    dil: Tuple[int, int, int] = (1, 1, 1)


def _layer_array(layers: Sequence[FcnLayer]):
    arr = (Layer * len(layers))()
    for i, L in enumerate(layers):
        _dev(L.w_bank, PACKED_DTYPE, "w_bank"); _dev(L.thr_lo, torch.int32, "thr_lo")
        _dev(L.thr_hi, torch.int32, "thr_hi")
        g = _geom(L.k, L.stride, L.pad, L.dil)
        if L.w_bank.numel() * 4 != tern_filter_bank_bytes(L.c_out, L.c_in, (g.k[0], g.k[1], g.k[2])):
            raise ValueError(f"layer {i}: w_bank size does not match (c_out, c_in, k)")
        if L.thr_lo.numel() != L.c_out or L.thr_hi.numel() != L.c_out:
            raise ValueError(f"layer {i}: cut points must have c_out entries")
        arr[i] = Layer(int(L.c_in), int(L.c_out), g, L.w_bank.data_ptr(), L.thr_lo.data_ptr(),
                       L.thr_hi.data_ptr())
    return arr


def tern_fcn_workspace_bytes(in_shape, layers: Sequence[FcnLayer]) -> int:
    arr = _layer_array(layers)
    return int(lib().tern_fcn_workspace_bytes(_dims(in_shape), arr, len(layers)))


def tern_fcn_forward(x: torch.Tensor, in_lo: torch.Tensor, in_hi: torch.Tensor,
                     layers: Sequence[FcnLayer], workspace: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None, return_layers: bool = False,
                     static_scratch: bool = False):
    """float32 [N][C0][D][H][W] -> packed output of the last module.  With return_layers, also a
    list of (packed tensor view, logical dims) for every module's output.  static_scratch=True
    calls tern_fcn_forward_static: no workspace, the activations between layers go to the
    library's fixed device array (return_layers then gives views of that array, valid until the
    next such call on this GPU)."""
    _dev(x, torch.float32, "x")
    if x.dim() != 5:
        raise ValueError("x must be [N][C0][D][H][W]")
    _dev(in_lo, torch.float32, "in_lo"); _dev(in_hi, torch.float32, "in_hi")
    if in_lo.numel() != x.shape[1] or in_hi.numel() != x.shape[1]:
        raise ValueError("input cut points must have C0 entries")
    arr = _layer_array(layers)
    need = int(lib().tern_fcn_workspace_bytes(_dims(x.shape), arr, len(layers)))
    if need == 0:
        raise TernError(-3, "tern_fcn_forward (invalid chain)")
    if static_scratch:
        if workspace is not None:
            raise ValueError("static_scratch takes no workspace")
    else:
        if workspace is None:
            workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
        _dev(workspace, torch.uint8, "workspace")
    # logical dims of every layer output
    dims_list: List[Tuple[int, ...]] = []
    cur = tuple(int(v) for v in x.shape)
    for L in layers:
        cur = tern_conv_out_dims(cur, L.c_out, L.k, L.stride, L.pad, L.dil)
        dims_list.append(cur)
    if out is None:
        out = _empty_packed(dims_list[-1], x.device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != tern_packed_bytes(dims_list[-1]):
        raise ValueError("out has the wrong size")
    od = Dims()
    ptrs = (C.c_void_p * len(layers))()
    if static_scratch:
        rc = lib().tern_fcn_forward_static(_ptr(x), _dims(x.shape), _ptr(in_lo), _ptr(in_hi), arr, len(layers),
                                           _ptr(out), C.byref(od), ptrs, _stream(x))
        _check(rc, "tern_fcn_forward_static")
    else:
        rc = lib().tern_fcn_forward(_ptr(x), _dims(x.shape), _ptr(in_lo), _ptr(in_hi), arr, len(layers),
                                    _ptr(workspace), workspace.numel(), _ptr(out), C.byref(od), ptrs,
                                    _stream(x))
        _check(rc, "tern_fcn_forward")
    if not return_layers:
        return out
    views = []
    if static_scratch:
        for i, dm in enumerate(dims_list):
            if i + 1 == len(layers):
                views.append((out, dm))
            else:
                shape = (dm[0], dm[2], dm[3], dm[4], 2, tern_words(dm[1]))
                views.append((torch.as_tensor(_DeviceWords(int(ptrs[i]), shape), device=x.device), dm))
        return out, views
    base = workspace.data_ptr()
    for i, dm in enumerate(dims_list):
        if i + 1 == len(layers):
            views.append((out, dm))
        else:
            off = int(ptrs[i]) - base
            nwords = tern_packed_bytes(dm) // 4
            v = workspace[off: off + nwords * 4].view(PACKED_DTYPE).view(
                dm[0], dm[2], dm[3], dm[4], 2, tern_words(dm[1]))
            views.append((v, dm))
    return out, views


def tern_static_scratch_bytes() -> int:
    """Size of the fixed device array behind tern_fcn_forward_static."""
    return int(lib().tern_static_scratch_bytes())


class _DeviceWords:
    """Device memory that no torch tensor owns (the library's fixed scratch array), described so
    that torch can view it without copying."""

    def __init__(self, ptr: int, shape):
        self.__cuda_array_interface__ = {"shape": tuple(int(v) for v in shape), "typestr": "<i4",
                                         "data": (int(ptr), False), "version": 2}


def tern_probe_valu(blocks: int, threads: int, iters: int, sink: torch.Tensor, variant: int = 0) -> None:
    """Diagnostic: enqueue the instruction probe (65 * iters vector instructions per lane);
    variant 0 = the kernels' spaced sequence, 1 = the same instructions unspaced, 2-13 = single
    opcodes and the binary word pair (see tern_tuning.h)."""
    _dev(sink, torch.int32, "sink")
    _check(lib().tern_probe_valu(int(blocks), int(threads), int(iters), int(variant), _ptr(sink), _stream(sink)),
           "tern_probe_valu")


def tern_set_option(option: int, value: int) -> None:
    """Tuning override (option numbers and values as in tern_option of the C header).  Results never
    depend on options."""
    _check(lib().tern_set_option(int(option), int(value)), "tern_set_option")


KERNEL_DIRECT, KERNEL_TILED, KERNEL_POINTWISE, KERNEL_PERSISTENT = 0, 1, 2, 3


def tern_last_launch() -> dict:
    """Plan of this thread's most recent convolution launch (see tern_tuning.h)."""
    info = (C.c_int32 * 8)()
    _check(lib().tern_last_launch(info), "tern_last_launch")
    keys = ("kernel", "voxels_per_lane", "channels_per_pass", "tap_split", "threads", "grid_x", "grid_y", "lds_bytes")
    return dict(zip(keys, (int(v) for v in info)))


# ---- U-Net plumbing ------------------------------------------------------------------------------
def _logical_dims(t: torch.Tensor, c: int):
    """Logical (n, c, d, h, w) of a packed tensor [N][D][H][W][2][Wd] holding c channels."""
    _dev(t, PACKED_DTYPE, "packed tensor")
    if t.dim() != 6 or t.shape[4] != 2 or t.shape[5] != tern_words(c):
        raise ValueError("packed tensor must be [N][D][H][W][2][ceil(C/32)]")
    return (int(t.shape[0]), int(c), int(t.shape[1]), int(t.shape[2]), int(t.shape[3]))


def tern_concat(sources, out_spatial=None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Gather-and-concatenate on packed tensors.  sources: sequence of (packed, channels[, up[,
    first]]) with up/first an int or three ints (defaults 1 and 0).  out_spatial: (d, h, w) of the
    output; default = the first source's upsampled extent minus its `first`.  Channels are laid
    out in the order of the sources."""
    srcs = []
    for s in sources:
        t, c = s[0], int(s[1])
        up = _t3(s[2]) if len(s) > 2 else (1, 1, 1)
        first = _t3(s[3]) if len(s) > 3 else (0, 0, 0)
        srcs.append((t, _logical_dims(t, c), up, first))
    if not srcs:
        raise ValueError("at least one source")
    if out_spatial is None:
        _, d0, up0, first0 = srcs[0]
        out_spatial = tuple(d0[2 + a] * up0[a] - first0[a] for a in range(3))
    n = srcs[0][1][0]
    c_total = sum(d[1] for _, d, _, _ in srcs)
    odims = (n, c_total) + tuple(int(v) for v in out_spatial)
    arr = (Source * len(srcs))()
    for i, (t, d, up, first) in enumerate(srcs):
        arr[i].packed = t.data_ptr()
        arr[i].dims = _dims(d)
        for a in range(3):
            arr[i].up[a] = up[a]
            arr[i].first[a] = first[a]
    if out is None:
        out = _empty_packed(odims, srcs[0][0].device)
    _dev(out, PACKED_DTYPE, "out")
    if out.numel() * 4 != tern_packed_bytes(odims):
        raise ValueError("out has the wrong size")
    _check(lib().tern_concat(arr, len(srcs), _dims(odims), _ptr(out), _stream(out)), "tern_concat")
    return out


def tern_conv3d_real(in_packed: torch.Tensor, c_in: int, w: torch.Tensor,
                     bias: Optional[torch.Tensor] = None, stride=1, pad=0, dil=1,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Packed ternary codes x float32 weights [C_out][C_in][kd][kh][kw] (+ bias) -> float32
    [N][C_out][Do][Ho][Wo]."""
    idims = _logical_dims(in_packed, c_in)
    _dev(w, torch.float32, "w")
    if w.dim() != 5 or w.shape[1] != c_in:
        raise ValueError("w must be [C_out][C_in][kd][kh][kw]")
    c_out = int(w.shape[0])
    k = tuple(int(x) for x in w.shape[2:])
    if bias is not None:
        _dev(bias, torch.float32, "bias")
        if bias.numel() != c_out:
            raise ValueError("bias must have C_out entries")
    odims = tern_conv_out_dims(idims, c_out, k, stride, pad, dil)
    if out is None:
        out = torch.empty(odims, dtype=torch.float32, device=w.device)
    _dev(out, torch.float32, "out")
    if tuple(out.shape) != tuple(odims):
        raise ValueError("out has the wrong shape")
    _check(lib().tern_conv3d_real(_ptr(in_packed), _dims(idims), _ptr(w),
                                  _ptr(bias) if bias is not None else None, c_out,
                                  _geom(k, stride, pad, dil), _ptr(out), _stream(out)),
           "tern_conv3d_real")
    return out


class NetModule:
    """One module of tern_net_forward: a fused ternary convolution whose input is the previous
    module's output, optionally upsampled (`up`) and followed by the centre-cropped output of
    module `skip_from`, optionally sum-pooled over `pool` (then w_bank is the bank of
    tern_digits_weights' output and the cut points refer to window sums)."""

    def __init__(self, c_out: int, w_bank: torch.Tensor, thr_lo: torch.Tensor, thr_hi: torch.Tensor,
                 k=3, stride=1, pad=0, dil=1, skip_from: int = -1, up=1, pool=1):
        _dev(w_bank, PACKED_DTYPE, "w_bank")
        _dev(thr_lo, torch.int32, "thr_lo")
        _dev(thr_hi, torch.int32, "thr_hi")
        self.c_out, self.w_bank, self.thr_lo, self.thr_hi = int(c_out), w_bank, thr_lo, thr_hi
        self.k, self.stride, self.pad, self.dil = _t3(k), _t3(stride), _t3(pad), _t3(dil)
        self.skip_from, self.up, self.pool = int(skip_from), _t3(up), _t3(pool)

    def as_struct(self) -> Module:
        m = Module(self.c_out, _geom(self.k, self.stride, self.pad, self.dil), self.w_bank.data_ptr(),
                   self.thr_lo.data_ptr(), self.thr_hi.data_ptr(), self.skip_from)
        for a in range(3):
            m.up[a] = self.up[a]
            m.pool[a] = self.pool[a]
        return m


def _module_array(mods):
    arr = (Module * len(mods))()
    for i, m in enumerate(mods):
        arr[i] = m.as_struct()
    return arr


def tern_net_workspace_bytes(in_shape, mods) -> int:
    return int(lib().tern_net_workspace_bytes(_dims(in_shape), _module_array(mods), len(mods)))


def tern_net_forward(x: torch.Tensor, in_lo: torch.Tensor, in_hi: torch.Tensor, mods,
                     head_w: Optional[torch.Tensor] = None, head_b: Optional[torch.Tensor] = None,
                     head_stride=1, head_pad=0, head_dil=1, workspace: Optional[torch.Tensor] = None,
                     head_out: Optional[torch.Tensor] = None, return_modules: bool = False):
    """Float input -> Eq. 6 -> modules with skips -> optional float-weight prediction layer.
    Returns the prediction maps (or None without a head) and, if return_modules, a list of
    (packed module output viewing the workspace, logical dims)."""
    _dev(x, torch.float32, "x")
    if x.dim() != 5:
        raise ValueError("x must be [N][C][D][H][W]")
    _dev(in_lo, torch.float32, "in_lo")
    _dev(in_hi, torch.float32, "in_hi")
    arr = _module_array(mods)
    need = int(lib().tern_net_workspace_bytes(_dims(x.shape), arr, len(mods)))
    if need == 0:
        raise TernError(-3, "tern_net_workspace_bytes (invalid module list)")
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    mod_ptr = (C.c_void_p * len(mods))()
    mod_dims = (Dims * len(mods))()
    hd = Dims()
    hk = Geom()
    head_c_out = 0
    if head_w is not None:
        _dev(head_w, torch.float32, "head_w")
        if head_w.dim() != 5:
            raise ValueError("head_w must be [C_out][C_in][kd][kh][kw]")
        head_c_out = int(head_w.shape[0])
        hk = _geom(tuple(int(v) for v in head_w.shape[2:]), head_stride, head_pad, head_dil)
        if head_b is not None:
            _dev(head_b, torch.float32, "head_b")
        if head_out is None:
            # extents of the last module, then of the head
            dims_list = _net_dims(x.shape, mods)
            ho = tern_conv_out_dims(dims_list[-1], head_c_out, tuple(int(v) for v in head_w.shape[2:]),
                                    head_stride, head_pad, head_dil)
            head_out = torch.empty(ho, dtype=torch.float32, device=x.device)
        _dev(head_out, torch.float32, "head_out")
    _check(lib().tern_net_forward(_ptr(x), _dims(x.shape), _ptr(in_lo), _ptr(in_hi), arr, len(mods),
                                  _ptr(head_w) if head_w is not None else None,
                                  _ptr(head_b) if head_b is not None else None, head_c_out, hk,
                                  _ptr(workspace), workspace.numel(),
                                  _ptr(head_out) if head_out is not None else None, C.byref(hd),
                                  mod_ptr, mod_dims, _stream(x)), "tern_net_forward")
    if not return_modules:
        return head_out
    views = []
    base = workspace.data_ptr()
    for i in range(len(mods)):
        d = mod_dims[i]
        dm = (d.n, d.c, d.d, d.h, d.w)
        nbytes = tern_packed_bytes(dm)
        off = mod_ptr[i] - base
        v = workspace[off:off + nbytes].view(PACKED_DTYPE).view(d.n, d.d, d.h, d.w, 2, tern_words(d.c))
        views.append((v, dm))
    return head_out, views


def _net_dims(in_shape, mods):
    """Logical dims of every module's output (host arithmetic mirroring the library's)."""
    out = []
    cur = tuple(int(v) for v in in_shape)
    for m in mods:
        n, c, d, h, w = cur
        d, h, w = d * m.up[0], h * m.up[1], w * m.up[2]
        if m.skip_from >= 0:
            c += out[m.skip_from][1]
        if max(m.pool) > 1:
            c, d, h, w = 64 * tern_words(c), d // m.pool[0], h // m.pool[1], w // m.pool[2]
        cur = tern_conv_out_dims((n, c, d, h, w), m.c_out, m.k, m.stride, m.pad, m.dil)
        out.append(cur)
    return out


def tern_count_codes(in_packed: torch.Tensor, c: int):
    """Per-channel (nonzero, negative) voxel counts of a packed tensor, two int64 tensors [C]."""
    dims = _logical_dims(in_packed, c)
    nz = torch.empty((c,), dtype=torch.int64, device=in_packed.device)
    ng = torch.empty((c,), dtype=torch.int64, device=in_packed.device)
    _check(lib().tern_count_codes(_ptr(in_packed), _dims(dims), _ptr(nz), _ptr(ng), _stream(in_packed)),
           "tern_count_codes")
    return nz, ng


# ---- host-side model preparation (numpy arrays in, numpy arrays out; no GPU involved) ----------
def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def tern_ternarize_filters(w):
    """float32 [C_out][...] host array -> (int8 codes of the same shape, float64 alpha[C_out])."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim < 2:
        raise ValueError("w must be [C_out][...]")
    codes = np.empty(w.shape, dtype=np.int8)
    alpha = np.empty(w.shape[0], dtype=np.float64)
    _check(lib().tern_ternarize_filters(_np_ptr(w), w.shape[0], w.size // w.shape[0], _np_ptr(codes),
                                        _np_ptr(alpha)), "tern_ternarize_filters")
    return codes, alpha


def tern_ternarize_filters_sparse(w, zeros: int):
    """As tern_ternarize_filters, with `zeros` entries of every filter (those of smallest magnitude)
    set to 0 instead of Eq. 4's threshold."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim < 2:
        raise ValueError("w must be [C_out][...]")
    codes = np.empty(w.shape, dtype=np.int8)
    alpha = np.empty(w.shape[0], dtype=np.float64)
    _check(lib().tern_ternarize_filters_sparse(_np_ptr(w), w.shape[0], w.size // w.shape[0], int(zeros),
                                               _np_ptr(codes), _np_ptr(alpha)), "tern_ternarize_filters_sparse")
    return codes, alpha


def tern_fold_thresholds(scale, shift, acc_bound: int):
    """Per-channel y = scale*acc + shift -> (lo int32[C], hi int32[C], negate uint8[C])."""
    import numpy as np
    scale = np.ascontiguousarray(scale, dtype=np.float64)
    shift = np.ascontiguousarray(shift, dtype=np.float64)
    if scale.ndim != 1 or scale.shape != shift.shape:
        raise ValueError("scale and shift must be 1-D arrays of the same length")
    c = scale.shape[0]
    lo = np.empty(c, np.int32); hi = np.empty(c, np.int32); neg = np.empty(c, np.uint8)
    _check(lib().tern_fold_thresholds(_np_ptr(scale), _np_ptr(shift), c, int(acc_bound), _np_ptr(lo),
                                      _np_ptr(hi), _np_ptr(neg)), "tern_fold_thresholds")
    return lo, hi, neg


def tern_fold_batchnorm(alpha, gamma, beta, mean, var, eps: float, acc_bound: int):
    import numpy as np
    arrs = [np.ascontiguousarray(v, dtype=np.float64) for v in (alpha, gamma, beta, mean, var)]
    c = arrs[0].shape[0]
    if any(a.ndim != 1 or a.shape[0] != c for a in arrs):
        raise ValueError("all per-channel arrays must be 1-D of the same length")
    lo = np.empty(c, np.int32); hi = np.empty(c, np.int32); neg = np.empty(c, np.uint8)
    _check(lib().tern_fold_batchnorm(*[_np_ptr(a) for a in arrs], float(eps), c, int(acc_bound),
                                     _np_ptr(lo), _np_ptr(hi), _np_ptr(neg)), "tern_fold_batchnorm")
    return lo, hi, neg


def tern_fold_avgpool(w, pool):
    """int8 ternary filters [C_out][C_in][kd][kh][kw] -> filters with every tap repeated pool
    times per axis, [C_out][C_in][kd*pd][kh*ph][kw*pw] (host arrays)."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.int8)
    if w.ndim != 5:
        raise ValueError("w must be [C_out][C_in][kd][kh][kw]")
    pool = _t3(pool)
    co, ci, kd, kh, kw = (int(x) for x in w.shape)
    out = np.empty((co, ci, kd * pool[0], kh * pool[1], kw * pool[2]), dtype=np.int8)
    parr = (C.c_int32 * 3)(*pool)
    _check(lib().tern_fold_avgpool(_np_ptr(w), co, ci, kd, kh, kw, parr, _np_ptr(out)),
           "tern_fold_avgpool")
    return out
