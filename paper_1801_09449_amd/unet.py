"""The paper's baseline U-Net (section 3, Table 1) prepared for tern_net_forward.

Preparation only: the layer list of the synthetic recipe (or of a trained model in the same form)
is turned into device-resident filter banks and a module array; the forward pass itself is one
call of the library (Eq. 6 on the float stack, fused ternary convolutions, upsample + skip
concatenation on packed planes, float-weight prediction layer).  2x2 average pooling is exact
either way it is done here: small problems fold it into the filters of the module that follows
(tern_fold_avgpool: taps repeated over the pooling window, stride multiplied: no extra launch,
four times the word pairs of the pooled convolution); large ones pool into two balanced-ternary
digits first (tern_pool_digits, one small launch) and convolve those (twice the word pairs).
"""
from typing import Dict, List, Sequence

import numpy as np
import torch

from . import binding as B


class UNetPlan:
    """Device-resident parameters of the network, prepared once."""

    def __init__(self, layers: Sequence[Dict], head_w, head_b, in_lo, in_hi, device="cuda"):
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        self.in_lo, self.in_hi = dev(np.asarray(in_lo, np.float32)), dev(np.asarray(in_hi, np.float32))
        saved: Dict[str, int] = {}
        self.mods: List[B.NetModule] = []          # pooling folded into the filters everywhere
        self._digit_mods: Dict[int, B.NetModule] = {}   # pooled modules in their two-digit form
        self._macs: Dict[int, float] = {}          # folded word-pair work per output voxel of such a module
        for i, L in enumerate(layers):
            w = np.ascontiguousarray(L["w"], dtype=np.int8)
            stride = tuple(int(v) for v in (L.get("stride") or (1, 1, 1)))
            pad = tuple(int(v) for v in (L.get("pad") or (0, 0, 0)))
            skip = saved[L["concat"]] if L.get("concat") else -1
            up = tuple(L.get("up") or (1, 1, 1))
            lo, hi = dev(np.asarray(L["lo"], np.int32)), dev(np.asarray(L["hi"], np.int32))
            pool = tuple(int(v) for v in L["pool"]) if L.get("pool") else None
            if pool and int(np.prod(pool)) <= 4 and max(pool) <= 4:
                dbank = B.tern_pack_filters(dev(B.tern_digits_weights(w)))
                k0 = tuple(int(v) for v in w.shape[2:])
                self._digit_mods[i] = B.NetModule(int(w.shape[0]), dbank, lo, hi, k=k0, stride=stride,
                                                  pad=pad, dil=1, skip_from=skip, up=up, pool=pool)
                self._macs[i] = float(w.size) * float(np.prod(pool))
            if pool:
                # pooling window P before a convolution of stride s and padding p: filters with
                # every tap repeated P times, stride s*P, padding p*P
                w = B.tern_fold_avgpool(w, pool)
                stride = tuple(a * b for a, b in zip(stride, pool))
                pad = tuple(a * b for a, b in zip(pad, pool))
            bank = B.tern_pack_filters(dev(w))
            kk = tuple(int(v) for v in w.shape[2:])
            self.mods.append(B.NetModule(int(w.shape[0]), bank, lo, hi, k=kk, stride=stride, pad=pad, dil=1,
                                         skip_from=skip, up=up))
            if L.get("save"):
                saved[L["save"]] = i
        self.head_w = dev(np.asarray(head_w, np.float32)) if head_w is not None else None
        self.head_b = dev(np.asarray(head_b, np.float32)) if head_b is not None else None
        self._ws = None
        self._chosen: Dict[tuple, List[B.NetModule]] = {}

    # A pooled module whose folded convolution is at least this many ternary MACs runs through
    # two digits instead (half the word pairs for one more small launch; measured break-even
    # between 1 and 3 GMAC on MI355X).
    DIGITS_FROM_MACS = 1.5e9

    def modules(self, in_shape) -> List[B.NetModule]:
        """The module list for an input of this shape (cached)."""
        key = tuple(int(v) for v in in_shape)
        if key not in self._chosen:
            dims = B._net_dims(key, self.mods)       # same extents either way
            mods = list(self.mods)
            for i, m in self._digit_mods.items():
                n, _, d, h, w = dims[i]
                if n * d * h * w * self._macs[i] >= self.DIGITS_FROM_MACS:
                    mods[i] = m
            self._chosen[key] = mods
        return self._chosen[key]

    def workspace(self, x: torch.Tensor) -> torch.Tensor:
        need = B.tern_net_workspace_bytes(x.shape, self.modules(x.shape))
        if self._ws is None or self._ws.numel() < need or self._ws.device != x.device:
            self._ws = torch.empty((need,), dtype=torch.uint8, device=x.device)
        return self._ws


def unet_forward(plan: UNetPlan, x: torch.Tensor, keep_layers: bool = False, out=None):
    """x: float32 [N][C0][D][H][W] on the GPU.  Returns the float32 prediction maps (and, if
    keep_layers, the list of (packed module output, channel count), views into the plan's
    workspace that the next call overwrites)."""
    res = B.tern_net_forward(x, plan.in_lo, plan.in_hi, plan.modules(x.shape), plan.head_w, plan.head_b,
                             workspace=plan.workspace(x), head_out=out, return_modules=keep_layers)
    if not keep_layers:
        return res
    pred, views = res
    return pred, [(v, dm[1]) for v, dm in views]
