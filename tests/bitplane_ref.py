"""Test-only numpy rendering of the paper's Eq. 9 on channel-packed bit-planes.

Written independently of both the C oracle and the GPU library: it exists to check that the
masked-Hamming form (two bit counts per word pair) equals the plain inner product, and to pin the
storage format (which bit is which channel, which plane is which) from a second implementation.
"""
import numpy as np


def np_pack(x: np.ndarray) -> np.ndarray:
    """int8 ternary [N][C][D][H][W] -> uint32 [N][D][H][W][2][ceil(C/32)], little-endian bits:
    channel c lives in bit c % 32 of word c // 32; plane 0 = (x != 0), plane 1 = (x < 0)."""
    n, c = x.shape[:2]
    words = (c + 31) // 32
    xm = np.moveaxis(x, 1, -1)                                  # [N][D][H][W][C]
    padw = [(0, 0)] * (xm.ndim - 1) + [(0, 32 * words - c)]
    planes = []
    for bits in ((xm != 0), (xm < 0)):
        b = np.pad(bits.astype(np.uint8), padw)
        by = np.packbits(b, axis=-1, bitorder="little")          # [...][4*words] bytes
        planes.append(np.ascontiguousarray(by).view("<u4"))      # [...][words]
    return np.stack(planes, axis=-2).astype(np.uint32)


def np_unpack(packed: np.ndarray, c: int) -> np.ndarray:
    words = packed.shape[-1]
    by = np.ascontiguousarray(packed.astype("<u4")).view(np.uint8)
    bits = np.unpackbits(by, axis=-1, bitorder="little")         # [...][2][32*words]
    m = bits[..., 0, :c].astype(np.int8)
    s = bits[..., 1, :c].astype(np.int8)
    x = m * (1 - 2 * s)
    return np.ascontiguousarray(np.moveaxis(x, -1, 1))


_POP8 = np.array([bin(i).count("1") for i in range(256)], dtype=np.int32)


def popcount32(a: np.ndarray) -> np.ndarray:
    a = a.astype(np.uint32)
    return (_POP8[a & 0xFF] + _POP8[(a >> 8) & 0xFF] + _POP8[(a >> 16) & 0xFF] + _POP8[(a >> 24) & 0xFF])


def hamming_conv3d(act_p: np.ndarray, w_p: np.ndarray, k, stride, pad, dil, with_counts=False):
    """Eq. 9 in the form  popc(M) - 2 popc(M & X),  M = mask_a & mask_w, X = sign_a ^ sign_w,
    summed over taps and channel words.  act_p [N][D][H][W][2][Wd], w_p [Co][kd][kh][kw][2][Wd].
    Out-of-volume voxels are all-zero words (mask 0)."""
    n, d, h, w = act_p.shape[:4]
    co = w_p.shape[0]
    od, oh, ow = [(x + 2 * p - dl * (kk - 1) - 1) // s + 1
                  for x, kk, s, p, dl in zip((d, h, w), k, stride, pad, dil)]
    ap = np.pad(act_p, [(0, 0), (pad[0], pad[0]), (pad[1], pad[1]), (pad[2], pad[2]), (0, 0), (0, 0)])
    acc_m = np.zeros((n, co, od, oh, ow), dtype=np.int32)
    acc_n = np.zeros_like(acc_m)
    for a in range(k[0]):
        for b in range(k[1]):
            for c in range(k[2]):
                sl = ap[:, a * dil[0]: a * dil[0] + (od - 1) * stride[0] + 1: stride[0],
                        b * dil[1]: b * dil[1] + (oh - 1) * stride[1] + 1: stride[1],
                        c * dil[2]: c * dil[2] + (ow - 1) * stride[2] + 1: stride[2]]
                ma, sa = sl[..., 0, :], sl[..., 1, :]             # [N][od][oh][ow][Wd]
                for o in range(co):
                    mw, sw = w_p[o, a, b, c, 0], w_p[o, a, b, c, 1]
                    M = ma & mw
                    Nn = M & (sa ^ sw)
                    acc_m[:, o] += popcount32(M).sum(axis=-1)
                    acc_n[:, o] += popcount32(Nn).sum(axis=-1)
    acc = acc_m - 2 * acc_n
    return (acc, acc_m, acc_n) if with_counts else acc
