"""Oracle for the pieces a U-Net needs around the ternary convolution (test infrastructure, not
the product): pooling, upsampling, skip concatenation and the full-precision prediction layer of
the paper's baseline architecture (section 3, Table 1), all on unpacked tensors, written as the
plain definitions in numpy.

Readings of the paper taken here (it names the operations but not their details):

* AvgPool 2x2 between two ternary modules.  The average of ternary codes is not ternary, but the
  convolution that follows is linear, so "pool, then convolve" is computed exactly on integers:
  pool_sum() returns window *sums* (= P x the average, P = window volume) and the following
  convolution runs on those small integers; its accumulator is P x the accumulator of the
  averaged tensor, which the cut points of the next activation absorb (scale a/P in Eq. 6's
  argument).  Nothing is rounded or re-ternarised at the pooling layer.
* Upsample 2x2: nearest neighbour (the only mode that keeps codes ternary).
* Skip connections: the stored encoder tensor is centre-cropped to the decoder tensor's extent
  (first voxel floor((X_skip - X)/2) per axis) and its channels are appended after the decoder's.
* Prediction layer: an ordinary cross-correlation of the ternary codes with real-valued weights
  plus a bias, evaluated in float64.

* A window sum of at most four ternary codes can also be written with two ternary digits,
  low + 3 * high (balanced ternary, unique on [-4, 4]); pool_digits() returns them.  Nothing in
  the paper: it is this build's way of keeping pooled tensors in the 2-bit format.

Pins: tests/test_unet_oracle.py (index-by-index brute force, hand-worked arrays, cross-check of
the real-weight convolution against a library convolution, pooling folded into a strided
convolution with repeated taps, digits: reconstruction of the sums and digit range on all 81
windows of four codes).
"""
from typing import Sequence, Tuple

import numpy as np


def pool_sum(x: np.ndarray, window: Tuple[int, int, int]) -> np.ndarray:
    """Window sums of x [N][C][D][H][W] over non-overlapping windows (pd, ph, pw); trailing
    voxels that do not fill a window are dropped.  Same integer dtype as x."""
    pd, ph, pw = window
    n, c, d, h, w = x.shape
    od, oh, ow = d // pd, h // ph, w // pw
    out = np.zeros((n, c, od, oh, ow), dtype=np.int64)
    for a in range(pd):
        for b in range(ph):
            for e in range(pw):
                out += x[:, :, a:od * pd:pd, b:oh * ph:ph, e:ow * pw:pw]
    return out.astype(x.dtype)


def pool_digits(x: np.ndarray, window: Tuple[int, int, int]):
    """Balanced-ternary digits of the window sums of ternary codes: (low, high) int8 tensors of
    pool_sum's shape with low + 3 * high == pool_sum(x, window) and both in {-1, 0, +1}; defined
    for windows of at most 4 voxels (sums in [-4, 4], where the representation exists and is
    unique).  Written as the definition: the high digit is the sum divided by 3 and rounded to
    the nearest integer, the low digit is what remains."""
    if window[0] * window[1] * window[2] > 4:
        raise ValueError("two digits cover sums in [-4, 4] only")
    s = pool_sum(np.asarray(x, dtype=np.int64), window)
    high = np.rint(s / 3.0).astype(np.int64)      # |s| <= 4: no ties at .5
    low = s - 3 * high
    return low.astype(np.int8), high.astype(np.int8)


def upsample_nearest(x: np.ndarray, factor: Tuple[int, int, int]) -> np.ndarray:
    """out[n][c][z][y][x] = in[n][c][z // fd][y // fh][x // fw]."""
    fd, fh, fw = factor
    return np.repeat(np.repeat(np.repeat(x, fd, axis=2), fh, axis=3), fw, axis=4)


def centre_crop(x: np.ndarray, spatial: Tuple[int, int, int]) -> np.ndarray:
    """The (d, h, w) window of x that starts at floor((X - x)/2) on every axis."""
    off = [(full - want) // 2 for full, want in zip(x.shape[2:], spatial)]
    if min(off) < 0:
        raise ValueError("crop larger than the tensor")
    return x[:, :, off[0]:off[0] + spatial[0], off[1]:off[1] + spatial[1], off[2]:off[2] + spatial[2]]


def concat_channels(parts: Sequence[np.ndarray]) -> np.ndarray:
    """Channel concatenation of tensors with equal N and spatial extents, in the order given."""
    return np.ascontiguousarray(np.concatenate(list(parts), axis=1))


def conv3d_real(act: np.ndarray, wgt: np.ndarray, bias, stride=(1, 1, 1), pad=(0, 0, 0),
                dil=(1, 1, 1)) -> np.ndarray:
    """float64 cross-correlation of integer codes act [N][C_in][D][H][W] with real weights
    [C_out][C_in][kd][kh][kw] plus bias [C_out] (or None); zero padding."""
    a = np.asarray(act, dtype=np.float64)
    w = np.asarray(wgt, dtype=np.float64)
    n, ci, d, h, wd = a.shape
    co, ci2, kd, kh, kw = w.shape
    if ci != ci2:
        raise ValueError("channel mismatch")
    ap = np.zeros((n, ci, d + 2 * pad[0], h + 2 * pad[1], wd + 2 * pad[2]))
    ap[:, :, pad[0]:pad[0] + d, pad[1]:pad[1] + h, pad[2]:pad[2] + wd] = a
    od = (d + 2 * pad[0] - dil[0] * (kd - 1) - 1) // stride[0] + 1
    oh = (h + 2 * pad[1] - dil[1] * (kh - 1) - 1) // stride[1] + 1
    ow = (wd + 2 * pad[2] - dil[2] * (kw - 1) - 1) // stride[2] + 1
    out = np.zeros((n, co, od, oh, ow))
    for ta in range(kd):
        for tb in range(kh):
            for tc in range(kw):
                z0, y0, x0 = ta * dil[0], tb * dil[1], tc * dil[2]
                patch = ap[:, :, z0:z0 + (od - 1) * stride[0] + 1:stride[0],
                           y0:y0 + (oh - 1) * stride[1] + 1:stride[1],
                           x0:x0 + (ow - 1) * stride[2] + 1:stride[2]]
                out += np.einsum("ncdhw,oc->nodhw", patch, w[:, :, ta, tb, tc])
    if bias is not None:
        out += np.asarray(bias, dtype=np.float64)[None, :, None, None, None]
    return out


def count_codes(x: np.ndarray):
    """Per-channel counts over batch and space of nonzero codes and of -1 codes of an integer
    tensor [N][C][...] (the zero fraction the paper discusses in section 4 is
    1 - nonzero / voxels).  Returns two int64 arrays [C]."""
    axes = (0,) + tuple(range(2, x.ndim))
    return (x != 0).sum(axis=axes).astype(np.int64), (x < 0).sum(axis=axes).astype(np.int64)


def unet_forward(x, in_lo, in_hi, layers, head_w, head_b):
    """The U-Net of Table 1 on unpacked tensors, module by module.

    x: float32 intensities, ternarised at (in_lo, in_hi) (Eq. 6).  layers: dicts as described by
    the synthetic recipe (w, k, lo, hi, pool, up, concat, save; optional stride/pad, default 1/0).  Every convolution is the integer
    oracle's (valid and stride 1 unless the layer says otherwise) and runs on the pooled sums where a pooling window is
    given.  Returns (list of per-module int8 codes, float64 prediction maps)."""
    from .tern_oracle import ConvGeom as geom, conv3d, threshold
    cur = threshold(np.ascontiguousarray(x, dtype=np.float32), in_lo, in_hi)
    saved, codes = {}, []
    for L in layers:
        if L.get("pool"):
            cur = pool_sum(cur, L["pool"])
        if L.get("up"):
            cur = upsample_nearest(cur, L["up"])
        if L.get("concat"):
            cur = concat_channels([cur, centre_crop(saved[L["concat"]], cur.shape[2:])])
        acc = conv3d(np.ascontiguousarray(cur), L["w"],
                     geom(L["k"], L.get("stride") or (1, 1, 1), L.get("pad") or (0, 0, 0), (1, 1, 1)))
        cur = threshold(acc, L["lo"], L["hi"])
        codes.append(cur)
        if L.get("save"):
            saved[L["save"]] = cur
    return codes, (conv3d_real(cur, head_w, head_b) if head_w is not None else None)
