"""Pins for the CPU oracle: every test checks it against something other than itself (brute
force, closed forms, a library routine, invariants, the paper's printed figures)."""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom
from tests.bitplane_ref import hamming_conv3d, np_pack, np_unpack, popcount32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_conv(act, wgt, k, stride, pad, dil):
    """Independent route: zero-pad the volume, gather the c = k^3 * C_in patch vector of each
    output, multiply element-wise with the flattened filter and sum (the inner product of two
    ternary vectors of length c, paper section 2)."""
    n, ci, d, h, w = act.shape
    co = wgt.shape[0]
    ap = np.pad(act.astype(np.int64), [(0, 0), (0, 0)] + [(p, p) for p in pad])
    od, oh, ow = [(x + 2 * p - dl * (kk - 1) - 1) // s + 1
                  for x, kk, s, p, dl in zip((d, h, w), k, stride, pad, dil)]
    out = np.zeros((n, co, od, oh, ow), dtype=np.int64)
    wf = wgt.astype(np.int64).reshape(co, -1)
    for b, z, y, x in itertools.product(range(n), range(od), range(oh), range(ow)):
        patch = ap[b, :,
                   z * stride[0]: z * stride[0] + dil[0] * (k[0] - 1) + 1: dil[0],
                   y * stride[1]: y * stride[1] + dil[1] * (k[1] - 1) + 1: dil[1],
                   x * stride[2]: x * stride[2] + dil[2] * (k[2] - 1) + 1: dil[2]].reshape(-1)
        out[b, :, z, y, x] = (wf * patch[None, :]).sum(axis=1)
    return out.astype(np.int32)


# ---- P1 brute force on tiny volumes --------------------------------------------------------
@pytest.mark.parametrize("k,stride,pad,dil,vol,ci,co", [
    ((3, 3, 3), (1, 1, 1), (1, 1, 1), (1, 1, 1), (4, 5, 3), 3, 2),
    ((3, 3, 3), (2, 2, 2), (1, 1, 1), (1, 1, 1), (5, 4, 5), 2, 3),
    ((3, 3, 3), (1, 1, 1), (2, 2, 2), (2, 2, 2), (5, 5, 5), 1, 2),
    ((3, 3, 3), (1, 2, 1), (3, 0, 1), (3, 1, 1), (5, 5, 4), 2, 2),
    ((1, 1, 1), (1, 1, 1), (0, 0, 0), (1, 1, 1), (3, 4, 5), 3, 4),
    ((1, 3, 2), (1, 1, 2), (0, 1, 0), (1, 2, 1), (3, 5, 5), 2, 2),
    ((3, 3, 3), (1, 1, 1), (0, 0, 0), (1, 1, 1), (3, 3, 3), 2, 1),
])
def test_p1_brute_force(k, stride, pad, dil, vol, ci, co):
    act = synth.ternary((2, ci) + vol, 0.3, 11, synth.T_ACT)
    wgt = synth.ternary((co, ci) + k, 0.4, 11, synth.T_WGT)
    got = oracle.conv3d(act, wgt, ConvGeom(k, stride, pad, dil))
    want = brute_conv(act, wgt, k, stride, pad, dil)
    assert got.shape == want.shape
    np.testing.assert_array_equal(got, want)


# ---- P2 Eq. 9 (masked Hamming distance) equals the inner product ---------------------------
@pytest.mark.parametrize("ci,co,stride,dil", [(32, 4, 1, 1), (33, 3, 2, 1), (70, 2, 1, 2), (5, 5, 1, 1)])
def test_p2_eq9_identity(ci, co, stride, dil):
    vol = (6, 5, 7)
    act = synth.ternary((1, ci) + vol, 0.4, 3, synth.T_ACT)
    wgt = synth.ternary((co, ci, 3, 3, 3), 0.5, 3, synth.T_WGT)
    g = ConvGeom.make(3, stride, dil, dil)
    want = oracle.conv3d(act, wgt, g)
    acc, acc_m, acc_n = hamming_conv3d(np_pack(act), np_pack(wgt), g.k, g.stride, g.pad, g.dil,
                                       with_counts=True)
    np.testing.assert_array_equal(acc, want)
    # P9: |acc| <= popc(M) and same parity
    assert np.all(np.abs(want) <= acc_m)
    assert np.all((want - acc_m) % 2 == 0)


# ---- P3 binary special case: Eq. 8 ----------------------------------------------------------
def test_p3_binary_special_case():
    ci, co, vol = 40, 3, (4, 4, 5)
    act = synth.ternary((1, ci) + vol, 0.0, 5, synth.T_ACT)      # no zeros: +-1 only
    wgt = synth.ternary((co, ci, 3, 3, 3), 0.0, 5, synth.T_WGT)
    assert np.all(act != 0) and np.all(wgt != 0)
    g = ConvGeom.make(3, 1, 0, 1)
    got = oracle.conv3d(act, wgt, g)
    c = 27 * ci
    # XOR of sign bits over the c-vector, counted without packing
    sa = (act < 0)
    sw = (wgt < 0)
    for o, z, y, x in itertools.product(range(co), range(2), range(2), range(3)):
        patch = sa[0, :, z:z + 3, y:y + 3, x:x + 3]
        ham = int(np.count_nonzero(patch ^ sw[o]))
        assert got[0, o, z, y, x] == c - 2 * ham


# ---- P4 zero invariants ---------------------------------------------------------------------
def test_p4_zero_invariants():
    act = synth.ternary((1, 6, 5, 5, 5), 0.3, 7, synth.T_ACT)
    wgt = synth.ternary((4, 6, 3, 3, 3), 0.5, 7, synth.T_WGT)
    g = ConvGeom.make()
    assert not oracle.conv3d(act, np.zeros_like(wgt), g).any()
    assert not oracle.conv3d(np.zeros_like(act), wgt, g).any()
    full = oracle.conv3d(act, wgt, g)
    w2 = wgt.copy(); w2[:, 2] = 0
    only2 = oracle.conv3d(np.ascontiguousarray(act[:, 2:3]), np.ascontiguousarray(wgt[:, 2:3]), g)
    np.testing.assert_array_equal(oracle.conv3d(act, w2, g), full - only2)


# ---- P5 antisymmetry ------------------------------------------------------------------------
def test_p5_antisymmetry_and_threshold_mirror():
    act = synth.ternary((2, 9, 6, 5, 4), 0.35, 9, synth.T_ACT)
    wgt = synth.ternary((5, 9, 3, 3, 3), 0.5, 9, synth.T_WGT)
    g = ConvGeom.make()
    acc = oracle.conv3d(act, wgt, g)
    np.testing.assert_array_equal(oracle.conv3d((-act).astype(np.int8), wgt, g), -acc)
    np.testing.assert_array_equal(oracle.conv3d(act, (-wgt).astype(np.int8), g), -acc)
    lo, hi = synth.threshold_pair(5, 9)
    code = oracle.threshold(acc, lo, hi)
    mirrored = oracle.threshold((-acc).astype(np.int32), (-hi).astype(np.int32), (-lo).astype(np.int32))
    np.testing.assert_array_equal(mirrored, -code)


# ---- P6 all-ones closed form (zero padding) -------------------------------------------------
def test_p6_all_ones_counts_in_bounds_taps():
    ci, vol = 7, (5, 6, 4)
    act = np.ones((1, ci) + vol, dtype=np.int8)
    wgt = np.ones((2, ci, 3, 3, 3), dtype=np.int8)
    acc = oracle.conv3d(act, wgt, ConvGeom.make())
    def taps(i, n):       # in-bounds taps along one axis for k=3, pad=1
        return 3 - (i == 0) - (i == n - 1)
    for z, y, x in itertools.product(range(vol[0]), range(vol[1]), range(vol[2])):
        want = ci * taps(z, vol[0]) * taps(y, vol[1]) * taps(x, vol[2])
        assert acc[0, 0, z, y, x] == want and acc[0, 1, z, y, x] == want
    assert acc[0, 0, 2, 2, 2] == 27 * ci and acc[0, 0, 0, 0, 0] == 8 * ci
    assert acc[0, 0, 0, 2, 2] == 18 * ci and acc[0, 0, 0, 0, 2] == 12 * ci


# ---- P7 delta kernels: orientation (cross-correlation), stride, dilation --------------------
@pytest.mark.parametrize("stride,dil", [(1, 1), (2, 1), (1, 2), (2, 3)])
def test_p7_delta_kernels(stride, dil):
    ci, vol = 3, (7, 6, 8)
    act = synth.ternary((1, ci) + vol, 0.3, 13, synth.T_ACT)
    pad = dil
    g = ConvGeom.make(3, stride, pad, dil)
    od, oh, ow = oracle.out_dims(act.shape, ci, g)
    ap = np.pad(act, [(0, 0), (0, 0)] + [(pad, pad)] * 3)
    for (a, b, c) in [(1, 1, 1), (0, 0, 0), (2, 1, 0), (0, 2, 1)]:
        wgt = np.zeros((ci, ci, 3, 3, 3), dtype=np.int8)
        for ch in range(ci):
            wgt[ch, ch, a, b, c] = 1
        acc = oracle.conv3d(act, wgt, g)
        # acc[z,y,x] = act[z*s - p + a*dil, ...]  (no kernel flip)
        want = ap[:, :, a * dil: a * dil + (od - 1) * stride + 1: stride,
                  b * dil: b * dil + (oh - 1) * stride + 1: stride,
                  c * dil: c * dil + (ow - 1) * stride + 1: stride]
        np.testing.assert_array_equal(acc, want.astype(np.int32))


# ---- P8 library cross-checks ----------------------------------------------------------------
@pytest.mark.parametrize("ci,co,vol,stride,pad,dil,k", [
    (16, 8, (9, 10, 11), 1, 1, 1, 3),
    (35, 6, (8, 9, 7), 2, 1, 1, 3),
    (12, 5, (9, 9, 9), 1, 2, 2, 3),
    (8, 4, (10, 7, 9), (2, 1, 2), (0, 2, 1), (1, 2, 1), (2, 3, 1)),
])
def test_p8_torch_conv3d_float64(ci, co, vol, stride, pad, dil, k):
    import torch
    g = ConvGeom.make(k, stride, pad, dil)
    act = synth.ternary((2, ci) + vol, 0.4, 17, synth.T_ACT)
    wgt = synth.ternary((co, ci) + g.k, 0.5, 17, synth.T_WGT)
    got = oracle.conv3d(act, wgt, g)
    ref = torch.nn.functional.conv3d(torch.from_numpy(act).double(), torch.from_numpy(wgt).double(),
                                     stride=g.stride, padding=g.pad, dilation=g.dil)
    np.testing.assert_array_equal(got, ref.numpy().astype(np.int32))


def test_p8_pointwise_kernel_is_matrix_product():
    ci, co, vol = 50, 20, (4, 5, 6)
    act = synth.ternary((1, ci) + vol, 0.4, 19, synth.T_ACT)
    wgt = synth.ternary((co, ci, 1, 1, 1), 0.5, 19, synth.T_WGT)
    got = oracle.conv3d(act, wgt, ConvGeom.make(1, 1, 0, 1))
    want = wgt.reshape(co, ci).astype(np.int32) @ act.reshape(ci, -1).astype(np.int32)
    np.testing.assert_array_equal(got.reshape(co, -1), want)


def test_points_variant_matches_full():
    c = synth.conv_case("t", 2, 10, 6, (6, 7, 5), stride=2, pad=1, seed=23)
    g = ConvGeom(c.k, c.stride, c.pad, c.dil)
    full = oracle.conv3d(c.act, c.wgt, g)
    idx = np.stack(np.unravel_index(np.arange(0, full.size, 7), full.shape), axis=1).astype(np.int32)
    got = oracle.conv3d_points(c.act, c.wgt, g, idx)
    np.testing.assert_array_equal(got, full.reshape(-1)[::7])


# ---- Eq. 6: strictness at ties --------------------------------------------------------------
def test_threshold_strict_outside_inclusive_band():
    v = np.arange(-4, 5, dtype=np.int32).reshape(1, 1, 9)
    code = oracle.threshold(v, np.array([-2], np.int32), np.array([1], np.int32))
    np.testing.assert_array_equal(code.reshape(-1), [-1, -1, 0, 0, 0, 0, 1, 1, 1])
    # lo == hi: only that value maps to 0
    code = oracle.threshold(v, np.array([0], np.int32), np.array([0], np.int32))
    np.testing.assert_array_equal(code.reshape(-1), [-1] * 4 + [0] + [1] * 4)
    # lo == hi + 1: empty zero band (a folded scale above 1 leaves no integer inside |y| <= 0.5)
    code = oracle.threshold(v, np.array([1], np.int32), np.array([0], np.int32))
    np.testing.assert_array_equal(code.reshape(-1), [-1] * 5 + [1] * 4)
    with pytest.raises(ValueError):
        oracle.threshold(v, np.array([2], np.int32), np.array([0], np.int32))
    # float form of Eq. 6 at the paper's cut points: x > 0.5 -> +1, |x| <= 0.5 -> 0, else -1
    x = np.array([-0.75, -0.5, -0.25, 0.0, 0.5, 0.5000001, 2.0, np.nan], np.float32).reshape(1, 1, -1)
    code = oracle.threshold(x, np.array([-0.5], np.float32), np.array([0.5], np.float32))
    np.testing.assert_array_equal(code.reshape(-1), [-1, 0, 0, 0, 0, 1, 1, 0])


def test_threshold_is_per_channel():
    v = np.tile(np.arange(-3, 4, dtype=np.int32), (2, 3, 1))
    lo = np.array([-1, 0, -3], np.int32); hi = np.array([1, 0, 3], np.int32)
    code = oracle.threshold(v, lo, hi)
    for ch in range(3):
        want = np.where(v[0, ch] > hi[ch], 1, np.where(v[0, ch] < lo[ch], -1, 0))
        np.testing.assert_array_equal(code[0, ch], want)
        np.testing.assert_array_equal(code[1, ch], want)


# ---- P11 storage format ---------------------------------------------------------------------
def test_p11_fig3_code_points():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "fig3_encoding.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for val, first, second in rows:
        val, first, second = int(val), int(first), int(second)
        p = oracle.pack(np.array([val], np.int8).reshape(1, 1, 1))
        mask, sign = int(p[0, 0, 0, 0]), int(p[0, 0, 1, 0])
        assert mask == 1 - second            # our mask plane is the complement of the zero flag
        if val != 0:
            assert sign == 1 - first         # our sign plane marks -1, the figure's marks +1
        else:
            assert sign == 0                 # canonical: no sign under a clear mask


@pytest.mark.parametrize("c", [1, 5, 31, 32, 33, 64, 70, 256])
def test_p11_pack_roundtrip_and_independent_packer(c):
    x = synth.ternary((2, c, 3, 4, 5), 0.4, 29, synth.T_ACT)
    p = oracle.pack(x)
    assert p.shape == (2, 3, 4, 5, 2, (c + 31) // 32) and p.dtype == np.uint32
    np.testing.assert_array_equal(p, np_pack(x))               # second implementation agrees
    np.testing.assert_array_equal(oracle.unpack(p, c), x)
    np.testing.assert_array_equal(np_unpack(p, c), x)
    assert np.all(p[..., 1, :] & ~p[..., 0, :] == 0)           # sign only under mask
    if c % 32:
        top = np.uint32((0xFFFFFFFF << (c % 32)) & 0xFFFFFFFF)
        assert np.all(p[..., :, -1] & top == 0)                # pad bits are zero
    # bit position: channel ch -> bit ch % 32 of word ch // 32
    one = np.zeros((1, c, 1, 1, 1), np.int8); ch = c - 1; one[0, ch] = -1
    q = oracle.pack(one)
    assert q[0, 0, 0, 0, 0, ch // 32] == np.uint32(1) << np.uint32(ch % 32)
    assert q[0, 0, 0, 0, 1, ch // 32] == np.uint32(1) << np.uint32(ch % 32)


def test_pack_rejects_non_ternary_and_unpack_rejects_fourth_code():
    with pytest.raises(ValueError):
        oracle.pack(np.array([2], np.int8).reshape(1, 1, 1))
    bad = np.zeros((1, 1, 2, 1), np.uint32); bad[0, 0, 1, 0] = 1     # sign without mask
    with pytest.raises(ValueError):
        oracle.unpack(bad, 3)
    stray = np.zeros((1, 1, 2, 1), np.uint32); stray[0, 0, 0, 0] = 1 << 5
    with pytest.raises(ValueError):
        oracle.unpack(stray, 3)


# ---- P13 generator statistics + metric convention -------------------------------------------
def test_p13_generator_statistics():
    n = 1 << 20
    for p0 in (0.3, 0.4, 0.5, 1.0 / 3.0):
        t = synth.ternary((n,), p0, 0, synth.T_ACT)
        z = np.count_nonzero(t == 0) / n
        assert abs(z - p0) < 3 * np.sqrt(p0 * (1 - p0) / n) + 1e-9
        pos = np.count_nonzero(t == 1) / n
        assert abs(pos - (1 - p0) / 2) < 4 * np.sqrt(0.25 / n)
    # order independence: a slice of a larger draw equals the draw at that offset
    u_all = synth.uniform01(1000, 5, 2)
    np.testing.assert_array_equal(u_all[100:200], synth.uniform01(100, 5, 2, offset=100))
    # different tensors are different streams
    assert np.any(synth.ternary((256,), 0.5, 0, synth.T_ACT) != synth.ternary((256,), 0.5, 0, synth.T_WGT))
    g = synth.gaussian((1 << 18,), 0, synth.T_F32)
    assert abs(float(g.mean())) < 0.01 and abs(float(g.std()) - 1.0) < 0.01
    assert abs(np.count_nonzero(np.abs(g) <= 0.5) / g.size - 0.3829) < 0.01


def test_p13_accumulator_statistics_cfg0_like():
    c = synth.conv_case("s", 1, 32, 8, 12, p0_w=0.5, p0_a=1.0 / 3.0, seed=0)
    acc = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    inner = acc[:, :, 1:-1, 1:-1, 1:-1].astype(np.float64)
    var = 27 * 32 * 0.5 * (2.0 / 3.0)
    assert abs(inner.mean()) < 1.5
    assert abs(inner.var() / var - 1.0) < 0.15


def test_mac_convention_matches_table1():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_mflops.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 8
    for _, ow, oh, kv, ci, co, printed in rows:
        macs = int(ow) * int(oh) * int(kv) * int(ci) * int(co)
        assert round(macs / 1e6) == int(printed)
    # the same convention as ConvCase.macs on a toy case
    c = synth.conv_case("m", 1, 4, 5, (6, 7, 8), seed=1)
    assert c.macs == 5 * 6 * 7 * 8 * 4 * 27
    assert synth.config2.__doc__  # recipe documented


def test_fcn_chain_matches_manual_chain():
    f = synth.config2(seed=2, vol=(8, 8, 8), channels=(4, 6, 6), strides=(1, 2, 1))
    layers = [dict(w=L["w"], geom=ConvGeom(L["k"], L["stride"], L["pad"], L["dil"]), lo=L["lo"], hi=L["hi"])
              for L in f.layers]
    codes, accs = oracle.fcn_forward(f.x, f.in_lo, f.in_hi, layers, keep_acc=True)
    cur = np.where(f.x > 0.5, 1, np.where(f.x < -0.5, -1, 0)).astype(np.int8)
    for L, code, acc in zip(f.layers, codes, accs):
        want_acc = brute_conv(cur, L["w"], L["k"], L["stride"], L["pad"], L["dil"])
        np.testing.assert_array_equal(acc, want_acc)
        cur = np.where(want_acc > L["hi"][None, :, None, None, None], 1,
                       np.where(want_acc < L["lo"][None, :, None, None, None], -1, 0)).astype(np.int8)
        np.testing.assert_array_equal(code, cur)
    assert codes[-1].shape == (1, 6, 4, 4, 4)
