"""The paper's baseline U-Net (section 3, Table 1) as a sequence of library calls on packed
activations.  Sequencing and argument marshalling only: every step runs in the HIP kernels.

  fp32 stack -> tern_threshold_pack (Eq. 6)
  each ternary module: [tern_concat of the upsampled tensor and the centre-cropped skip tensor]
                       -> tern_conv3d with fused activation and re-packing
  2x2 average pooling is not a step of its own: it is folded into the filters of the module that
  follows (tern_fold_avgpool: taps repeated, stride multiplied), which is exact
  prediction layer: tern_conv3d_real (float weights on ternary codes).
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
        self.mods: List[Dict] = []
        for L in layers:
            w = np.ascontiguousarray(L["w"], dtype=np.int8)
            stride = (1, 1, 1)
            if L.get("pool"):
                w = B.tern_fold_avgpool(w, L["pool"])
                stride = tuple(int(p) for p in L["pool"])
            self.mods.append(dict(
                bank=B.tern_pack_filters(dev(w)), c_in=int(w.shape[1]), c_out=int(w.shape[0]),
                k=tuple(int(v) for v in w.shape[2:]), stride=stride,
                lo=dev(np.asarray(L["lo"], np.int32)), hi=dev(np.asarray(L["hi"], np.int32)),
                concat=L.get("concat"), up=tuple(L.get("up") or (1, 1, 1)), save=L.get("save")))
        self.head_w = dev(np.asarray(head_w, np.float32))
        self.head_b = dev(np.asarray(head_b, np.float32))


def unet_forward(plan: UNetPlan, x: torch.Tensor, keep_layers: bool = False):
    """x: float32 [N][C0][D][H][W] on the GPU.  Returns the float32 prediction maps (and, if
    keep_layers, the list of packed module outputs with their channel counts)."""
    cur = B.tern_threshold_pack(x, plan.in_lo, plan.in_hi)
    c_cur = int(x.shape[1])
    saved, kept = {}, []
    for m in plan.mods:
        if m["concat"]:
            skip, c_skip = saved[m["concat"]]
            up = m["up"]
            spatial = tuple(int(cur.shape[1 + a]) * up[a] for a in range(3))
            first = tuple((int(skip.shape[1 + a]) - spatial[a]) // 2 for a in range(3))
            cur = B.tern_concat([(cur, c_cur, up), (skip, c_skip, 1, first)], out_spatial=spatial)
            c_cur += c_skip
        cur = B.tern_conv3d(cur, c_cur, m["bank"], m["c_out"], m["k"], m["stride"], 0, 1,
                            thr_lo=m["lo"], thr_hi=m["hi"])
        c_cur = m["c_out"]
        if m["save"]:
            saved[m["save"]] = (cur, c_cur)
        if keep_layers:
            kept.append((cur, c_cur))
    pred = B.tern_conv3d_real(cur, c_cur, plan.head_w, plan.head_b)
    return (pred, kept) if keep_layers else pred
