"""Pins for the U-Net oracle pieces (pooling sums, nearest upsampling, centre crop + concat,
real-weight prediction convolution) and for the host helper that folds average pooling into the
following convolution.  None of these tests needs a GPU."""
import os

import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom


def rnd_tern(shape, seed, p0=0.3):
    return synth.ternary(shape, p0, seed, synth.T_ACT)


def test_pool_sum_hand_example_and_brute_force():
    x = np.array([[1, -1, 0], [0, 1, 1], [1, 1, 1]], np.int8).reshape(1, 1, 1, 3, 3)
    np.testing.assert_array_equal(oracle.pool_sum(x, (1, 2, 2)).reshape(-1), [1])   # 1-1+0+1, rest dropped
    x = rnd_tern((2, 3, 5, 7, 6), 3)
    got = oracle.pool_sum(x, (2, 3, 2))
    assert got.shape == (2, 3, 2, 2, 3) and got.dtype == np.int8
    for n in range(2):
        for c in range(3):
            for z in range(2):
                for y in range(2):
                    for xx in range(3):
                        want = sum(int(x[n, c, 2 * z + a, 3 * y + b, 2 * xx + e])
                                   for a in range(2) for b in range(3) for e in range(2))
                        assert got[n, c, z, y, xx] == want


def test_pool_sum_is_window_volume_times_library_average():
    import torch
    x = rnd_tern((1, 4, 4, 6, 8), 5)
    avg = torch.nn.functional.avg_pool3d(torch.from_numpy(x.astype(np.float64)), (1, 2, 2)).numpy()
    np.testing.assert_array_equal(oracle.pool_sum(x, (1, 2, 2)), np.rint(avg * 4).astype(np.int8))
    assert np.abs(avg * 4 - np.rint(avg * 4)).max() == 0


def test_upsample_nearest_index_by_index():
    x = rnd_tern((1, 2, 2, 3, 4), 7)
    up = oracle.upsample_nearest(x, (1, 2, 3))
    assert up.shape == (1, 2, 2, 6, 12)
    for z in range(2):
        for y in range(6):
            for xx in range(12):
                assert (up[0, :, z, y, xx] == x[0, :, z, y // 2, xx // 3]).all()
    import torch
    lib = torch.nn.functional.interpolate(torch.from_numpy(x.astype(np.float32)), scale_factor=(1, 2, 3),
                                          mode="nearest").numpy()
    np.testing.assert_array_equal(up, lib.astype(np.int8))


def test_centre_crop_offsets_and_concat_order():
    x = np.arange(1 * 1 * 1 * 5 * 8, dtype=np.int8).reshape(1, 1, 1, 5, 8)
    c = oracle.centre_crop(x, (1, 2, 3))
    # offsets floor((5-2)/2) = 1 and floor((8-3)/2) = 2
    np.testing.assert_array_equal(c[0, 0, 0], x[0, 0, 0, 1:3, 2:5])
    np.testing.assert_array_equal(oracle.centre_crop(x, (1, 5, 8)), x)
    with pytest.raises(ValueError):
        oracle.centre_crop(x, (1, 6, 8))
    a, b = rnd_tern((2, 3, 1, 2, 2), 1), rnd_tern((2, 5, 1, 2, 2), 2)
    cat = oracle.concat_channels([a, b])
    assert cat.shape == (2, 8, 1, 2, 2)
    np.testing.assert_array_equal(cat[:, :3], a)
    np.testing.assert_array_equal(cat[:, 3:], b)


@pytest.mark.parametrize("stride,pad,dil", [((1, 1, 1), (0, 0, 0), (1, 1, 1)), ((1, 2, 1), (0, 1, 2), (1, 1, 2)),
                                            ((2, 1, 2), (1, 0, 1), (1, 2, 1))])
def test_conv3d_real_against_library_and_integer_oracle(stride, pad, dil):
    import torch
    act = rnd_tern((2, 5, 4, 7, 6), 11)
    w = synth.gaussian((3, 5, 2, 3, 3), 11, synth.T_F32)
    b = synth.gaussian((3,), 12, synth.T_F32)
    got = oracle.conv3d_real(act, w, b, stride, pad, dil)
    lib = torch.nn.functional.conv3d(torch.from_numpy(act.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                     torch.from_numpy(b.astype(np.float64)), stride, pad, dil).numpy()
    np.testing.assert_allclose(got, lib, rtol=0, atol=1e-12)
    # with ternary "real" weights and no bias it is the integer convolution, exactly
    wi = synth.ternary((3, 5, 2, 3, 3), 0.5, 13, synth.T_WGT)
    exact = oracle.conv3d(act, wi, ConvGeom((2, 3, 3), stride, pad, dil))
    np.testing.assert_array_equal(oracle.conv3d_real(act, wi, None, stride, pad, dil), exact.astype(np.float64))


def test_conv3d_real_single_tap_hand_example():
    act = np.array([1, -1, 0, 1], np.int8).reshape(1, 4, 1, 1, 1)
    w = np.array([[0.5, 0.25, 8.0, -2.0]], np.float64).reshape(1, 4, 1, 1, 1)
    out = oracle.conv3d_real(act, w, np.array([0.125]))
    assert out.reshape(-1)[0] == 0.5 - 0.25 - 2.0 + 0.125


@pytest.mark.parametrize("vol,k,pool,pad", [((1, 11, 10), (1, 3, 3), (1, 2, 2), (0, 0, 0)),
                                            ((6, 9, 7), (2, 3, 1), (2, 2, 3), (0, 0, 0)),
                                            ((1, 9, 9), (1, 1, 1), (1, 2, 2), (0, 0, 0)),
                                            ((4, 8, 10), (3, 3, 3), (1, 2, 2), (1, 1, 1))])
def test_pool_then_conv_equals_strided_conv_with_repeated_taps(vol, k, pool, pad):
    """The identity behind tern_fold_avgpool, checked on the integer oracle alone and then on the
    library's host helper."""
    import paper_1801_09449_amd as T
    x = rnd_tern((2, 3) + vol, 21)
    w = synth.ternary((4, 3) + k, 0.4, 21, synth.T_WGT)
    pooled = oracle.conv3d(oracle.pool_sum(x, pool), w, ConvGeom(k, (1, 1, 1), pad, (1, 1, 1)))
    rep = np.repeat(np.repeat(np.repeat(w, pool[0], axis=2), pool[1], axis=3), pool[2], axis=4)
    kk = tuple(a * b for a, b in zip(k, pool))
    folded = oracle.conv3d(x, np.ascontiguousarray(rep),
                           ConvGeom(kk, pool, tuple(a * b for a, b in zip(pad, pool)), (1, 1, 1)))
    np.testing.assert_array_equal(folded, pooled)
    if not os.path.exists(T.lib_path()):
        from paper_1801_09449_amd import build
        build.build()
    np.testing.assert_array_equal(T.tern_fold_avgpool(w, pool), rep)


def test_count_codes_hand_example():
    x = np.array([[[1, 0, -1], [0, 0, -1]], [[-1, 1, 1], [0, -1, 0]]], np.int8).reshape(2, 2, 1, 1, 3)
    nz, ng = oracle.count_codes(x)
    # channel 0: items (1,0,-1) and (-1,1,1); channel 1: (0,0,-1) and (0,-1,0)
    np.testing.assert_array_equal(nz, [5, 2])
    np.testing.assert_array_equal(ng, [2, 2])
    x = rnd_tern((3, 5, 4, 6, 7), 9, p0=0.4)
    nz, ng = oracle.count_codes(x)
    for c in range(5):
        assert nz[c] == sum(int(v != 0) for v in x[:, c].reshape(-1))
        assert ng[c] == sum(int(v < 0) for v in x[:, c].reshape(-1))
    # the generator's zero fraction shows up
    assert abs(1 - nz.sum() / x.size - 0.4) < 0.03


def test_unet_chain_shapes_follow_valid_arithmetic():
    u = synth.unet_table1(seed=3, width_div=16, size=(76, 68), slices=5)
    codes, pred = oracle.unet_forward(u.x, u.in_lo, u.in_hi, u.layers, u.head_w, u.head_b)
    hw = [c.shape[3:] for c in codes]
    # 76x68 -> 74x66 -> 72x64 -> 70x62 -> pool 35x31 -> 33x29 -> 31x27 -> pool 15x13 -> 13x11 -> 13x11
    # -> pool 6x5 -> 6x5 -> up 12x10 -> 10x8 -> 8x6 -> up 16x12 -> 14x10 -> 12x8 -> up 24x16 -> 22x14 -> 20x12
    assert hw == [(74, 66), (72, 64), (70, 62), (33, 29), (31, 27), (13, 11), (13, 11), (6, 5),
                  (10, 8), (8, 6), (14, 10), (12, 8), (22, 14), (20, 12)]
    assert all(c.shape[2] == 1 for c in codes)
    assert pred.shape == (1, 2, 1, 18, 10)
    # every module keeps a healthy mix of codes (the cut-point recipe does not collapse)
    for c in codes:
        z = np.mean(c == 0)
        assert 0.1 < z < 0.8


def test_unet_table1_extents_where_the_table_is_consistent():
    """Rows 1, 2, 9-12 of Table 1 print output sizes that follow from valid 3x3 convolutions,
    2x2 pooling (floor) and 2x upsampling; the recipe reproduces them."""
    sizes = {}
    h, w = 236, 172
    chain = [("c", 3), ("c", 3), ("c", 3), ("p",), ("c", 3), ("c", 3), ("p",), ("c", 3), ("c", 1), ("p",),
             ("c", 1), ("u",), ("c", 3), ("c", 3), ("u",), ("c", 3), ("c", 3), ("u",), ("c", 3), ("c", 3)]
    li = 0
    for op in chain:
        if op[0] == "c":
            li += 1
            h, w = h - op[1] + 1, w - op[1] + 1
            sizes[li] = (h, w)
        elif op[0] == "p":
            h, w = h // 2, w // 2
        else:
            h, w = 2 * h, 2 * w
    printed = {1: (234, 170), 2: (232, 168), 9: (50, 34), 10: (48, 32), 11: (94, 62), 12: (92, 60)}
    for k, v in printed.items():
        assert sizes[k] == v


def test_pool_digits_reconstruct_the_sums_on_every_window_of_four_codes():
    """All 3^4 windows of four ternary codes: low + 3 * high is the window sum and both digits are
    ternary; the representation is unique, so this pins the function completely."""
    import itertools
    combos = np.array(list(itertools.product((-1, 0, 1), repeat=4)), dtype=np.int8)     # [81][4]
    x = combos.reshape(81, 1, 1, 2, 2)                                                # one 2x2 window each
    low, high = oracle.pool_digits(x, (1, 2, 2))
    assert low.shape == high.shape == (81, 1, 1, 1, 1)
    s = combos.astype(np.int64).sum(axis=1)
    np.testing.assert_array_equal(low.reshape(-1).astype(np.int64) + 3 * high.reshape(-1), s)
    assert set(np.unique(low)) <= {-1, 0, 1} and set(np.unique(high)) <= {-1, 0, 1}
    # hand-worked: 2 = -1 + 3, -4 = -1 - 3, 3 = 0 + 3, 1 = 1 + 0
    for codes, want in [((1, 1, 0, 0), (-1, 1)), ((-1, -1, -1, -1), (-1, -1)), ((1, 1, 1, 0), (0, 1)),
                        ((1, 0, 0, 0), (1, 0)), ((1, -1, 0, 0), (0, 0))]:
        l, h = oracle.pool_digits(np.array(codes, np.int8).reshape(1, 1, 1, 2, 2), (1, 2, 2))
        assert (int(l.item()), int(h.item())) == want
    # other window shapes, several channels, trailing voxels dropped like pool_sum
    x = synth.ternary((2, 5, 3, 5, 7), 0.3, 3, synth.T_ACT)
    for win in [(1, 2, 2), (2, 2, 1), (1, 1, 3), (1, 1, 1), (2, 1, 2)]:
        l, h = oracle.pool_digits(x, win)
        np.testing.assert_array_equal(l.astype(np.int64) + 3 * h, oracle.pool_sum(x.astype(np.int64), win))
    with pytest.raises(ValueError):
        oracle.pool_digits(x, (2, 2, 2))
