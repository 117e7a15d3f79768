"""Seeded synthetic inputs for the ternary-convolution tests and benchmark.

This module only draws numbers.  It holds none of the method's arithmetic (no convolution, no
packing, no thresholding of accumulators) and is the one piece of code that both the CPU oracle's
tests and the GPU library's tests/benchmark use, so that both sides see identical inputs.

Generator: counter based and order independent.  Element `i` of tensor `tensor_id` under `seed`
is derived from splitmix64(seed ^ (tensor_id << 56) ^ i); the top 53 bits give u in [0, 1).
Ternary value: 0 if u < p0, +1 if u < p0 + (1 - p0)/2, else -1.

The tensors stand in for the CT volumes and trained weights the paper used (section 3), which are
not available: only shapes and zero fractions are taken from the paper (weights about half zeros,
section 2 after Eq. 9; activations roughly unit normal through the +-0.5 activation of Eq. 6,
about 38 % zeros).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

T_ACT, T_WGT, T_THR, T_F32 = 1, 2, 3, 4

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """Finaliser of the splitmix64 generator applied element-wise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x.astype(np.uint64) + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    return np.uint64((int(seed) ^ (int(tensor_id) << 56)) & 0xFFFFFFFFFFFFFFFF)


def uniform01(count: int, seed: int, tensor_id: int, offset: int = 0) -> np.ndarray:
    """count doubles in [0,1), element i drawn from counter offset+i."""
    out = np.empty(count, dtype=np.float64)
    key = _key(seed, tensor_id)
    step = 1 << 22
    for s in range(0, count, step):
        e = min(count, s + step)
        idx = np.arange(offset + s, offset + e, dtype=np.uint64)
        out[s:e] = (splitmix64(idx ^ key) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return out


def ternary(shape, p0: float, seed: int, tensor_id: int) -> np.ndarray:
    """int8 tensor with P(0) = p0 and P(+1) = P(-1) = (1 - p0)/2, C-order counter."""
    count = int(np.prod(shape, dtype=np.int64))
    out = np.empty(count, dtype=np.int8)
    step = 1 << 22
    for s in range(0, count, step):
        e = min(count, s + step)
        u = uniform01(e - s, seed, tensor_id, offset=s)
        out[s:e] = np.where(u < p0, 0, np.where(u < p0 + (1.0 - p0) / 2.0, 1, -1)).astype(np.int8)
    return out.reshape(shape)


def uniform_int(count: int, lo: int, hi: int, seed: int, tensor_id: int, offset: int = 0) -> np.ndarray:
    """count integers uniform in [lo, hi] (inclusive) as int64."""
    u = uniform01(count, seed, tensor_id, offset)
    return (np.floor(u * (hi - lo + 1)).astype(np.int64) + lo).clip(lo, hi)


def gaussian(shape, seed: int, tensor_id: int) -> np.ndarray:
    """float32 N(0,1) samples (Box-Muller on counters 2i and 2i+1)."""
    count = int(np.prod(shape, dtype=np.int64))
    u = uniform01(2 * count, seed, tensor_id).reshape(count, 2)
    r = np.sqrt(-2.0 * np.log(1.0 - u[:, 0]))  # 1-u in (0,1]
    return (r * np.cos(2.0 * np.pi * u[:, 1])).astype(np.float32).reshape(shape)


def threshold_pair(c: int, seed: int, tensor_id: int = T_THR, lo: int = -8, hi: int = 8
                   ) -> Tuple[np.ndarray, np.ndarray]:
    """Two integer cut points per channel: t1, t2 i.i.d. uniform in [lo, hi]; (min, max)."""
    t = uniform_int(2 * c, lo, hi, seed, tensor_id).reshape(c, 2)
    return t.min(axis=1).astype(np.int32), t.max(axis=1).astype(np.int32)


def bn_like_thresholds(c_out: int, fan_in_taps: int, c_in: int, p_w: float, p_a: float,
                       seed: int, tensor_id: int) -> Tuple[np.ndarray, np.ndarray]:
    """Integer cut points imitating "batch-norm to about unit normal, then +-0.5" for a layer
    whose accumulator has standard deviation sigma = sqrt(taps * c_in * p_w * p_a) (p_w, p_a =
    nonzero fractions).  Per channel a = (1 + 0.1 u)/sigma, b = 0.1 g (u uniform[-1,1], g normal);
    the real cut points (+-0.5 - b)/a are rounded to the integers that decide an integer
    accumulator identically: hi = floor((0.5 - b)/a), lo = ceil((-0.5 - b)/a).  This is an input
    recipe, not part of the method."""
    sigma = np.sqrt(fan_in_taps * c_in * p_w * p_a)
    u = uniform01(c_out, seed, tensor_id) * 2.0 - 1.0
    uu = uniform01(2 * c_out, seed, tensor_id, offset=1 << 20).reshape(c_out, 2)
    g = np.sqrt(-2.0 * np.log(1.0 - uu[:, 0])) * np.cos(2.0 * np.pi * uu[:, 1])
    a = (1.0 + 0.1 * u) / sigma
    b = 0.1 * g
    hi = np.floor((0.5 - b) / a).astype(np.int64)
    lo = np.ceil((-0.5 - b) / a).astype(np.int64)
    lo = np.minimum(lo, hi)
    return lo.astype(np.int32), hi.astype(np.int32)


@dataclass
class ConvCase:
    """One single-layer workload: unpacked int8 tensors plus geometry and cut points."""
    name: str
    act: np.ndarray            # int8 [N][C_in][D][H][W]
    wgt: np.ndarray            # int8 [C_out][C_in][kd][kh][kw]
    k: Tuple[int, int, int]
    stride: Tuple[int, int, int]
    pad: Tuple[int, int, int]
    dil: Tuple[int, int, int]
    lo: np.ndarray             # int32 [C_out]
    hi: np.ndarray             # int32 [C_out]
    meta: Dict = field(default_factory=dict)

    @property
    def out_spatial(self) -> Tuple[int, int, int]:
        return tuple((x + 2 * p - dl * (kk - 1) - 1) // s + 1
                     for x, kk, s, p, dl in zip(self.act.shape[2:], self.k, self.stride, self.pad, self.dil))

    @property
    def macs(self) -> int:
        """Nominal dense multiply-accumulate count: outputs x kernel volume x C_in (the
        convention of the paper's Table 1: zeros and padded taps are counted)."""
        od, oh, ow = self.out_spatial
        return (self.act.shape[0] * self.wgt.shape[0] * od * oh * ow * self.act.shape[1]
                * self.k[0] * self.k[1] * self.k[2])


def conv_case(name: str, n: int, c_in: int, c_out: int, vol, k=3, stride=1, pad=1, dil=1,
              p0_w: float = 0.5, p0_a: float = 1.0 / 3.0, seed: int = 0,
              thr_range: Tuple[int, int] = (-8, 8)) -> ConvCase:
    t3 = lambda v: (v,) * 3 if isinstance(v, int) else tuple(v)
    vol, k, stride, pad, dil = t3(vol), t3(k), t3(stride), t3(pad), t3(dil)
    act = ternary((n, c_in) + vol, p0_a, seed, T_ACT)
    wgt = ternary((c_out, c_in) + k, p0_w, seed, T_WGT)
    lo, hi = threshold_pair(c_out, seed, T_THR, *thr_range)
    return ConvCase(name, act, wgt, k, stride, pad, dil, lo, hi,
                    dict(p0_w=p0_w, p0_a=p0_a, seed=seed))


def config0(seed: int = 0) -> ConvCase:
    """C_in = C_out = 32, 24^3, 3^3, stride 1, pad 1; weights P(0)=0.5, activations uniform."""
    return conv_case("cfg0", 1, 32, 32, 24, p0_w=0.5, p0_a=1.0 / 3.0, seed=seed)


def config1(seed: int = 0, vol=64) -> ConvCase:
    """C_in = C_out = 64, 64^3, 3^3; weight zeros 0.5, activation zeros 0.4; cut points in [-8,8]."""
    return conv_case("cfg1", 1, 64, 64, vol, p0_w=0.5, p0_a=0.4, seed=seed)


def config3(seed: int = 0, vol=32, n: int = 2) -> ConvCase:
    """C_in = C_out = 256, batch 2, 32^3; weight zeros 0.6, activation zeros 0.5."""
    return conv_case("cfg3", n, 256, 256, vol, p0_w=0.6, p0_a=0.5, seed=seed)


def config4_cases(seed: int = 0, vol=96) -> List[ConvCase]:
    """C_in = C_out = 64 on vol^3: 3^3 kernels at dilation 1,2,3 (pad = dilation) and 1^3 kernels
    (pad 0), each at weight zero fractions 0.3, 0.5, 0.7; activation zeros 0.4."""
    out = []
    for p0 in (0.3, 0.5, 0.7):
        for dil in (1, 2, 3):
            out.append(conv_case(f"cfg4_k3_d{dil}_pw{p0}", 1, 64, 64, vol, k=3, pad=dil, dil=dil,
                                 p0_w=p0, p0_a=0.4, seed=seed))
        out.append(conv_case(f"cfg4_k1_pw{p0}", 1, 64, 64, vol, k=1, pad=0, dil=1,
                             p0_w=p0, p0_a=0.4, seed=seed))
    return out


@dataclass
class FcnCase:
    """Encoder workload: float intensities, input cut points, and per-layer tensors."""
    name: str
    x: np.ndarray              # float32 [N][C0][D][H][W]
    in_lo: np.ndarray          # float32 [C0]
    in_hi: np.ndarray          # float32 [C0]
    layers: List[Dict]         # each: w int8, k/stride/pad/dil triples, lo/hi int32

    @property
    def macs(self) -> int:
        total, sp = 0, self.x.shape[2:]
        for L in self.layers:
            sp = tuple((x + 2 * p - dl * (kk - 1) - 1) // s + 1
                       for x, kk, s, p, dl in zip(sp, L["k"], L["stride"], L["pad"], L["dil"]))
            total += (self.x.shape[0] * L["w"].shape[0] * sp[0] * sp[1] * sp[2] * L["w"].shape[1]
                      * L["k"][0] * L["k"][1] * L["k"][2])
        return total


def config2(seed: int = 0, vol=(128, 128, 64), channels=(16, 32, 32, 64, 64, 128),
            strides=(1, 2, 1, 2, 1, 2), c0: int = 1) -> FcnCase:
    """Six 3^3 layers, channels 1-16-32-32-64-64-128, stride 2 at layers 2, 4, 6; N(0,1)
    intensities ternarised at +-0.5; weight zeros 0.5; cut points from bn_like_thresholds with
    nonzero fractions 0.5 (weights) and 0.617 (activations).  c0: input channels (1 in the
    configuration; more for tests of chains whose first layer sees several)."""
    x = gaussian((1, c0) + tuple(vol), seed, T_F32)
    layers, c_in = [], c0
    for li, (c_out, s) in enumerate(zip(channels, strides), start=1):
        w = ternary((c_out, c_in, 3, 3, 3), 0.5, seed, T_WGT + 8 * li)
        lo, hi = bn_like_thresholds(c_out, 27, c_in, 0.5, 0.617, seed, T_THR + 8 * li)
        layers.append(dict(w=w, k=(3, 3, 3), stride=(s,) * 3, pad=(1, 1, 1), dil=(1, 1, 1),
                           lo=lo, hi=hi))
        c_in = c_out
    return FcnCase("cfg2", x, np.full(c0, -0.5, np.float32), np.full(c0, 0.5, np.float32), layers)


@dataclass
class UNetCase:
    """The paper's baseline U-Net (section 3, Table 1) with synthetic ternary weights.

    layers: one dict per ternary module, in order, each with
      w (int8 [C_out][C_in][kd][kh][kw]), lo/hi (int32 [C_out], cut points on the integer
      accumulator the module produces, pooling factor included), and what happens to the
      module's input before the convolution:
        pool   : (pd, ph, pw) average-pooling window applied to the incoming tensor, or None;
        up     : nearest-neighbour upsampling factors applied to the incoming tensor, or None;
        concat : name of a saved tensor that is centre-cropped to the (upsampled) incoming
                 extent and appended channel-wise, or None;
      and save: name under which the module's output codes are kept for a later skip, or None.
    head_w / head_b: float32 weights [classes][C][1][3][3] and bias of the prediction layer.
    """
    name: str
    x: np.ndarray
    in_lo: np.ndarray
    in_hi: np.ndarray
    layers: List[Dict]
    head_w: np.ndarray
    head_b: np.ndarray


def unet_table1(seed: int = 0, n: int = 1, size=(236, 172), slices: int = 15, width_div: int = 1,
                classes: int = 2) -> UNetCase:
    """Layer list of Table 1: #1 is a 3x3x15 convolution over the stack of `slices` neighbouring
    slices (one input channel, depth extent collapses to 1), #2-#14 are 2-D 3x3 (1x1 at #7, #8)
    valid convolutions with 2x2 average pooling before #4, #6, #8 and 2x upsampling plus skip
    concatenation (#6 -> #9, #4 -> #11, #2 -> #13) before #9, #11, #13.  Channel counts
    32-64-64-128-128-256-256-256-256-128-128-64-64-64, divided by width_div.  Input: N(0,1)
    intensities (zero mean, unit variance as in the paper's preprocessing) ternarised at +-0.5;
    weights: half zeros; cut points from bn_like_thresholds with the pooling factor counted as
    extra taps.  Spatial extents follow from valid-convolution arithmetic on `size`."""
    ch = [max(1, c // width_div) for c in (32, 64, 64, 128, 128, 256, 256, 256, 256, 128, 128, 64, 64, 64)]
    k2 = [3, 3, 3, 3, 3, 3, 1, 1, 3, 3, 3, 3, 3, 3]
    pool = {4: (1, 2, 2), 6: (1, 2, 2), 8: (1, 2, 2)}
    save = {2: "s2", 4: "s4", 6: "s6"}
    concat = {9: "s6", 11: "s4", 13: "s2"}
    x = gaussian((n, 1, slices) + tuple(size), seed, T_F32)
    layers, c_in = [], 1
    for li in range(1, 15):
        c_out = ch[li - 1]
        cin_l = c_in + (ch[{9: 6, 11: 4, 13: 2}[li] - 1] if li in concat else 0)
        k = (slices, 3, 3) if li == 1 else (1, k2[li - 1], k2[li - 1])
        w = ternary((c_out, cin_l) + k, 0.5, seed, T_WGT + 8 * li)
        pvol = int(np.prod(pool[li])) if li in pool else 1
        lo, hi = bn_like_thresholds(c_out, k[0] * k[1] * k[2] * pvol, cin_l, 0.5, 0.617, seed, T_THR + 8 * li)
        layers.append(dict(w=w, k=k, lo=lo, hi=hi, pool=pool.get(li), concat=concat.get(li),
                           up=(1, 2, 2) if li in concat else None, save=save.get(li)))
        c_in = c_out
    head_w = (gaussian((classes, c_in, 1, 3, 3), seed, T_F32 + 8 * 15) * 0.1).astype(np.float32)
    head_b = (gaussian((classes,), seed, T_F32 + 8 * 16) * 0.1).astype(np.float32)
    return UNetCase("unet_table1", x, np.array([-0.5], np.float32), np.array([0.5], np.float32),
                    layers, head_w, head_b)
