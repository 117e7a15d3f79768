"""GPU parity for the U-Net pieces around the ternary convolution: gather/concat on packed
tensors, 2-D (single-plane) convolutions, average pooling folded into the next convolution, the
real-weight prediction layer, and the whole Table 1 network, each against the CPU oracle on the
same seeded inputs.  Integer and bit results must match exactly; the float prediction layer
within the bound its summation order implies."""
import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    import paper_1801_09449_amd as T
    from tests import gpu_util
    T.lib()
    assert torch.cuda.is_available()
    return gpu_util


def tern(shape, seed, p0=0.35, tid=synth.T_ACT):
    return synth.ternary(shape, p0, seed, tid)


def gpu_pack(G, x):
    import paper_1801_09449_amd as T
    return T.tern_pack(G.dev(x))


# ---- tern_concat --------------------------------------------------------------------------------
@pytest.mark.parametrize("c,vol,up", [(5, (2, 3, 4), (1, 2, 2)), (33, (1, 5, 7), (1, 2, 2)), (64, (3, 4, 5), (2, 1, 3)),
                                      (70, (2, 2, 2), (3, 3, 3))])
def test_upsample_nearest(G, c, vol, up):
    import paper_1801_09449_amd as T
    x = tern((2, c) + vol, 5)
    got = T.tern_concat([(gpu_pack(G, x), c, up)])
    np.testing.assert_array_equal(G.words(got), oracle.pack(oracle.upsample_nearest(x, up)))


def test_centre_crop(G):
    import paper_1801_09449_amd as T
    x = tern((2, 40, 3, 9, 12), 6)
    want = oracle.centre_crop(x, (2, 4, 7))
    got = T.tern_concat([(gpu_pack(G, x), 40, 1, (0, 2, 2))], out_spatial=(2, 4, 7))
    np.testing.assert_array_equal(G.words(got), oracle.pack(np.ascontiguousarray(want)))


@pytest.mark.parametrize("chans", [(32, 32), (64, 64), (20, 50), (1, 1), (31, 33, 7), (96, 5, 40, 3), (7,) * 8])
def test_concat_any_channel_counts(G, chans):
    """Word-aligned and unaligned channel counts, up to the maximum number of sources."""
    import paper_1801_09449_amd as T
    parts = [tern((2, c, 2, 5, 6), 10 + i) for i, c in enumerate(chans)]
    got = T.tern_concat([(gpu_pack(G, p), p.shape[1]) for p in parts])
    want = oracle.pack(oracle.concat_channels(parts))
    assert got.shape[-1] == (sum(chans) + 31) // 32
    np.testing.assert_array_equal(G.words(got), want)


def test_decoder_step_upsample_crop_concat(G):
    """The decoder step of the U-Net: upsampled tensor first, centre-cropped skip tensor after."""
    import paper_1801_09449_amd as T
    low = tern((2, 48, 1, 6, 5), 31)
    skip = tern((2, 20, 1, 15, 13), 32)
    up = oracle.upsample_nearest(low, (1, 2, 2))
    want = oracle.concat_channels([up, oracle.centre_crop(skip, up.shape[2:])])
    first = tuple((s - u) // 2 for s, u in zip(skip.shape[2:], up.shape[2:]))
    got = T.tern_concat([(gpu_pack(G, low), 48, (1, 2, 2)), (gpu_pack(G, skip), 20, 1, first)],
                        out_spatial=up.shape[2:])
    np.testing.assert_array_equal(G.words(got), oracle.pack(want))


def test_concat_rejects_bad_arguments(G):
    import paper_1801_09449_amd as T
    a = gpu_pack(G, tern((1, 8, 2, 4, 4), 1))
    b = gpu_pack(G, tern((2, 8, 2, 4, 4), 2))
    with pytest.raises(T.TernError) as e:
        T.tern_concat([(a, 8), (b, 8)], out_spatial=(2, 4, 4))          # batch mismatch
    assert e.value.status == -3
    with pytest.raises(T.TernError) as e:
        T.tern_concat([(a, 8, 1, (0, 1, 0))], out_spatial=(2, 4, 4))    # crop runs past the source
    assert e.value.status == -3
    with pytest.raises(T.TernError) as e:
        T.tern_concat([(a, 8)] * 9, out_spatial=(2, 4, 4))              # too many sources
    assert e.value.status == -3


# ---- 2-D convolutions (single output plane) ---------------------------------------------------------
@pytest.mark.parametrize("n,ci,co,hw,k,stride", [(1, 32, 32, (17, 23), (1, 3, 3), 1), (3, 64, 40, (20, 19), (1, 3, 3), 1),
                                                 (2, 15, 32, (30, 26), (1, 3, 3), 1), (1, 128, 64, (33, 9), (1, 1, 1), 1),
                                                 (4, 8, 16, (21, 22), (1, 6, 6), (1, 2, 2)),
                                                 (5, 70, 33, (9, 40), (1, 3, 3), (1, 2, 1))])
def test_conv2d_single_plane(G, n, ci, co, hw, k, stride):
    """D = 1: a lane's voxels are stacked along y, and batch items are folded into planes for the
    packed output.  Both output modes against the oracle."""
    c = synth.conv_case("c2d", n, ci, co, (1,) + hw, k=k, stride=stride, pad=0, seed=n + ci)
    acc, packed = G.run_case(c)
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    np.testing.assert_array_equal(acc, want)
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(want, c.lo, c.hi)))


def test_conv_depth_one_kernel_on_a_volume_with_batch(G):
    """kd = 1 on D > 1 with N > 1 (planes independent: batch folded into depth), padded in-plane."""
    c = synth.conv_case("kd1", 3, 40, 24, (5, 12, 11), k=(1, 3, 3), pad=(0, 1, 1), seed=8)
    acc, packed = G.run_case(c)
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    np.testing.assert_array_equal(acc, want)
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(want, c.lo, c.hi)))


def test_first_layer_of_table1_stack_kernel(G):
    """Row #1 of Table 1: one input channel, kernel spanning the whole stack of 15 slices."""
    c = synth.conv_case("row1", 2, 1, 32, (15, 20, 22), k=(15, 3, 3), pad=0, seed=4)
    acc, packed = G.run_case(c)
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    assert want.shape[2] == 1
    np.testing.assert_array_equal(acc, want)
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(want, c.lo, c.hi)))


# ---- average pooling folded into the next convolution ----------------------------------------------
@pytest.mark.parametrize("vol,k,pool", [((1, 23, 21), (1, 3, 3), (1, 2, 2)), ((6, 10, 9), (3, 3, 3), (2, 2, 2)),
                                        ((1, 13, 11), (1, 1, 1), (1, 2, 2))])
def test_avgpool_folded_into_conv(G, vol, k, pool):
    import paper_1801_09449_amd as T
    x = tern((2, 24) + vol, 17)
    w = tern((40, 24) + k, 18, 0.5, synth.T_WGT)
    lo, hi = synth.threshold_pair(40, 19, lo=-6, hi=6)
    want = oracle.conv3d(oracle.pool_sum(x, pool), w, ConvGeom(k, (1, 1, 1), (0, 0, 0), (1, 1, 1)))
    wf = T.tern_fold_avgpool(w, pool)
    bank = T.tern_pack_filters(G.dev(wf))
    xp = gpu_pack(G, x)
    acc = T.tern_conv3d(xp, 24, bank, 40, wf.shape[2:], pool, 0, 1)
    np.testing.assert_array_equal(acc.cpu().numpy(), want)
    codes = T.tern_conv3d(xp, 24, bank, 40, wf.shape[2:], pool, 0, 1, thr_lo=G.dev(lo), thr_hi=G.dev(hi))
    np.testing.assert_array_equal(G.words(codes), oracle.pack(oracle.threshold(want, lo, hi)))


# ---- prediction layer ------------------------------------------------------------------------------
def real_conv_bound(w, b):
    """|fp32 result - exact| <= terms * 2^-24 * (|bias| + sum|w| of the filter), per output channel."""
    terms = w[0].size + 1
    mass = np.abs(w.astype(np.float64)).reshape(w.shape[0], -1).sum(axis=1) + np.abs(b.astype(np.float64))
    return terms * 2.0 ** -24 * mass


@pytest.mark.parametrize("ci,co,vol,k,stride,pad,dil", [(64, 2, (1, 20, 18), (1, 3, 3), 1, 0, 1),
                                                        (37, 5, (4, 6, 7), (3, 3, 3), (1, 2, 1), (1, 0, 2), (1, 1, 2)),
                                                        (8, 1, (3, 3, 3), (1, 1, 1), 1, 0, 1),
                                                        (300, 2, (3, 4, 5), (3, 3, 3), 1, 1, 1),     # filters too large for LDS
                                                        (130, 7, (2, 9, 70), (1, 3, 3), 1, (0, 1, 1), 1)])
def test_conv3d_real(G, ci, co, vol, k, stride, pad, dil):
    import paper_1801_09449_amd as T
    t3 = lambda v: (v,) * 3 if isinstance(v, int) else tuple(v)
    x = tern((2, ci) + vol, 23)
    w = synth.gaussian((co, ci) + k, 23, synth.T_F32)
    b = synth.gaussian((co,), 24, synth.T_F32)
    want = oracle.conv3d_real(x, w, b, t3(stride), t3(pad), t3(dil))
    got = T.tern_conv3d_real(gpu_pack(G, x), ci, G.dev(w), G.dev(b), stride, pad, dil).cpu().numpy()
    assert got.shape == want.shape and got.dtype == np.float32
    bound = real_conv_bound(w, b)[None, :, None, None, None]
    assert (np.abs(got.astype(np.float64) - want) <= bound).all()
    # without bias
    got0 = T.tern_conv3d_real(gpu_pack(G, x), ci, G.dev(w), None, stride, pad, dil).cpu().numpy()
    want0 = oracle.conv3d_real(x, w, None, t3(stride), t3(pad), t3(dil))
    assert (np.abs(got0.astype(np.float64) - want0) <= bound).all()
    # ternary-valued float weights: every partial sum is a small integer, the result is exact
    wi = tern((co, ci) + k, 25, 0.5, synth.T_WGT)
    exact = oracle.conv3d(x, wi, ConvGeom(k, t3(stride), t3(pad), t3(dil)))
    goti = T.tern_conv3d_real(gpu_pack(G, x), ci, G.dev(wi.astype(np.float32)), None, stride, pad, dil).cpu().numpy()
    np.testing.assert_array_equal(goti, exact.astype(np.float32))


# ---- code statistics ---------------------------------------------------------------------------------
@pytest.mark.parametrize("n,c,vol", [(1, 1, (1, 1, 1)), (2, 5, (3, 5, 7)), (1, 33, (4, 9, 11)), (3, 64, (2, 8, 8)),
                                     (1, 100, (5, 13, 6)), (2, 256, (3, 4, 5)), (1, 16, (40, 64, 70))])
def test_count_codes(G, n, c, vol):
    import paper_1801_09449_amd as T
    x = tern((n, c) + vol, 71, p0=0.45)
    nz, ng = T.tern_count_codes(gpu_pack(G, x), c)
    want_nz, want_ng = oracle.count_codes(x)
    np.testing.assert_array_equal(nz.cpu().numpy(), want_nz)
    np.testing.assert_array_equal(ng.cpu().numpy(), want_ng)


def test_count_codes_ignores_sign_under_clear_mask_and_repeats(G):
    import torch
    import paper_1801_09449_amd as T
    x = tern((1, 40, 3, 6, 5), 72)
    p = gpu_pack(G, x).clone()
    p[..., 1, :] = -1                      # every sign bit set, also under clear mask bits
    want_nz, _ = oracle.count_codes(x)
    for _ in range(2):                     # the call overwrites its outputs: same answer twice
        nz, ng = T.tern_count_codes(p, 40)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(nz.cpu().numpy(), want_nz)
        np.testing.assert_array_equal(ng.cpu().numpy(), want_nz)     # every nonzero now reads as -1


# ---- pooled convolutions through two balanced-ternary digits -----------------------------------------
def digits_of(words, c):
    """(low, high) int8 tensors [N][c][D][H][W] from a packed two-digit tensor (numpy words
    [N][D][H][W][2][2*wd])."""
    wd = (c + 31) // 32
    m, s = words[..., 0, :], words[..., 1, :]
    out = []
    for which in (0, 1):
        mm, ss = m[..., which::2], s[..., which::2]                      # [N][D][H][W][wd]
        bits = np.arange(32, dtype=np.uint32)
        mb = ((mm[..., None] >> bits) & 1).reshape(mm.shape[:-1] + (32 * wd,))[..., :c]
        sb = ((ss[..., None] >> bits) & 1).reshape(ss.shape[:-1] + (32 * wd,))[..., :c]
        code = mb.astype(np.int8) * (1 - 2 * sb.astype(np.int8))
        out.append(np.moveaxis(code, -1, 1))
    return out


@pytest.mark.parametrize("c,vol,win", [(5, (3, 6, 8), (1, 2, 2)), (32, (1, 7, 9), (1, 2, 2)), (70, (4, 5, 6), (2, 2, 1)),
                                       (64, (2, 4, 9), (1, 1, 3)), (33, (3, 3, 3), (1, 1, 1)), (96, (2, 8, 8), (2, 1, 2))])
def test_pool_digits(G, c, vol, win):
    import paper_1801_09449_amd as T
    x = synth.ternary((2, c) + vol, 0.3, c + vol[0], synth.T_ACT)
    got, c2 = T.tern_pool_digits(T.tern_pack(G.dev(x)), c, win)
    assert c2 == 64 * ((c + 31) // 32)
    words = G.words(got)
    low, high = digits_of(words, c)
    want_low, want_high = oracle.pool_digits(x, win)
    np.testing.assert_array_equal(low, want_low)
    np.testing.assert_array_equal(high, want_high)
    # canonical packing: no sign bit without its mask bit, padding channels empty
    assert not (words[..., 1, :] & ~words[..., 0, :]).any()
    if c % 32:
        assert not (words[..., 0, -2:] >> np.uint32(c % 32)).any()


@pytest.mark.parametrize("ci,co,vol,k,win", [(64, 40, (1, 30, 26), (1, 3, 3), (1, 2, 2)), (40, 33, (6, 12, 10), (3, 3, 3), (1, 2, 2)),
                                             (128, 64, (2, 21, 18), (1, 3, 3), (1, 2, 2)), (256, 48, (1, 16, 20), (1, 1, 1), (1, 2, 2)),
                                             (32, 16, (4, 9, 9), (2, 3, 1), (2, 1, 2))])
def test_conv_on_pooled_digits_equals_conv_on_window_sums(G, ci, co, vol, k, win):
    """tern_pool_digits + tern_conv3d_digits against the oracle's convolution of the window sums:
    int32 accumulators and fused packed output, both channel-block widths."""
    import paper_1801_09449_amd as T
    x = synth.ternary((2, ci) + vol, 0.35, ci + co, synth.T_ACT)
    w = synth.ternary((co, ci) + k, 0.5, ci + co, synth.T_WGT)
    pvol = win[0] * win[1] * win[2]
    lo, hi = synth.bn_like_thresholds(co, int(np.prod(k)) * pvol, ci, 0.5, 0.65, ci, synth.T_THR)
    pooled = np.ascontiguousarray(oracle.pool_sum(x, win))      # int8 sums in [-4, 4]
    geom = ConvGeom(k, (1, 1, 1), (0, 0, 0), (1, 1, 1))
    want_acc = oracle.conv3d(pooled, w, geom)
    want_packed = oracle.pack(oracle.threshold(want_acc, lo, hi))
    dig, c2 = T.tern_pool_digits(T.tern_pack(G.dev(x)), ci, win)
    bank = T.tern_pack_filters(G.dev(T.tern_digits_weights(w)))
    try:
        for cb in (0, 16, 32):
            T.tern_set_option(3, cb)
            acc = T.tern_conv3d(dig, c2, bank, co, k=k, stride=1, pad=0, dil=1, digits=True)
            packed = T.tern_conv3d(dig, c2, bank, co, k=k, stride=1, pad=0, dil=1, thr_lo=G.dev(lo),
                                   thr_hi=G.dev(hi), digits=True)
            np.testing.assert_array_equal(acc.cpu().numpy(), want_acc)
            np.testing.assert_array_equal(G.words(packed), want_packed)
    finally:
        T.tern_set_option(3, 0)
    # the same through the matrix cores: the two digits of a value become its 4-bit float code,
    # the bank is that of the undoubled weights
    mbank = T.tern_expand_filters(G.dev(w), "f4")
    acc = T.tern_conv3d(dig, c2, mbank, co, k=k, stride=1, pad=0, dil=1, digits=True, mfma="f4")
    packed = T.tern_conv3d(dig, c2, mbank, co, k=k, stride=1, pad=0, dil=1, thr_lo=G.dev(lo), thr_hi=G.dev(hi),
                           digits=True, mfma="f4")
    np.testing.assert_array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_array_equal(G.words(packed), want_packed)


def test_two_digit_input_through_the_direct_kernel(G):
    """A dilation whose halo tile no LDS holds: tern_conv3d_digits runs on the direct kernel (odd
    words count three times) and must still equal the convolution of the window sums; the matrix
    route refuses such a halo."""
    import paper_1801_09449_amd as T
    ci, co, win, k = 40, 33, (1, 2, 2), (2, 3, 3)
    x = synth.ternary((1, ci, 110, 18, 18), 0.35, 611, synth.T_ACT)
    w = synth.ternary((co, ci) + k, 0.5, 612, synth.T_WGT)
    lo, hi = synth.bn_like_thresholds(co, 18 * 4, ci, 0.5, 0.65, ci, synth.T_THR)
    pooled = np.ascontiguousarray(oracle.pool_sum(x, win))
    geom = ConvGeom(k, (1, 1, 1), (0, 1, 1), (100, 1, 1))
    want_acc = oracle.conv3d(pooled, w, geom)
    assert want_acc.shape == (1, co, 10, 9, 9)
    want_packed = oracle.pack(oracle.threshold(want_acc, lo, hi))
    dig, c2 = T.tern_pool_digits(T.tern_pack(G.dev(x)), ci, win)
    bank = T.tern_pack_filters(G.dev(T.tern_digits_weights(w)))
    kw = dict(k=k, stride=1, pad=(0, 1, 1), dil=(100, 1, 1), digits=True)
    acc = T.tern_conv3d(dig, c2, bank, co, **kw)
    packed = T.tern_conv3d(dig, c2, bank, co, thr_lo=G.dev(lo), thr_hi=G.dev(hi), **kw)
    np.testing.assert_array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_array_equal(G.words(packed), want_packed)
    with pytest.raises(T.TernError) as e:
        T.tern_conv3d(dig, c2, T.tern_expand_filters(G.dev(w), "f4"), co, mfma="f4", **kw)
    assert e.value.status == -2


# ---- the whole network -----------------------------------------------------------------------------
def run_unet(G, u):
    import torch
    from paper_1801_09449_amd import unet
    plan = unet.UNetPlan(u.layers, u.head_w, u.head_b, u.in_lo, u.in_hi)
    pred, kept = unet.unet_forward(plan, G.dev(u.x), keep_layers=True)
    torch.cuda.synchronize()
    return pred.cpu().numpy(), [G.words(t) for t, _ in kept], kept, plan


def check_unet(G, u):
    """Runs the network and compares every module with the oracle; returns the plan."""
    pred, kept, kept_dev, plan = run_unet(G, u)
    codes, want_pred = oracle.unet_forward(u.x, u.in_lo, u.in_hi, u.layers, u.head_w, u.head_b)
    assert len(kept) == len(codes) == 14
    for li, (got, want) in enumerate(zip(kept, codes), start=1):
        np.testing.assert_array_equal(got, oracle.pack(want), err_msg=f"module #{li}")
    # zero fraction per module from the library's statistics = the oracle's
    import paper_1801_09449_amd as T
    for (t, c), want in zip(kept_dev, codes):
        nz, ng = T.tern_count_codes(t, c)
        want_nz, want_ng = oracle.count_codes(want)
        np.testing.assert_array_equal(nz.cpu().numpy(), want_nz)
        np.testing.assert_array_equal(ng.cpu().numpy(), want_ng)
    bound = real_conv_bound(u.head_w, u.head_b)[None, :, None, None, None]
    assert pred.shape == want_pred.shape
    assert (np.abs(pred.astype(np.float64) - want_pred) <= bound).all()
    return plan


def test_unet_reduced(G):
    """Narrow network on small stacks, batch of 3: every module's packed output, bit for bit."""
    check_unet(G, synth.unet_table1(seed=5, n=3, width_div=8, size=(84, 76), slices=5))
    check_unet(G, synth.unet_table1(seed=6, n=1, width_div=3, size=(92, 100), slices=15))


def test_unet_many_stacks_take_the_two_kernel_first_module(G):
    """Four full-size stacks, narrow channels: module #1 has more output voxels than the fused
    gather-and-convolve kernel is used for, so its taps are gathered to memory and convolved by the
    pointwise kernel over five words (one stack takes the fused kernel, see the full-size test)."""
    check_unet(G, synth.unet_table1(seed=7, n=4, width_div=8))


def test_unet_reduced_with_every_pooled_module_through_two_digits(G, monkeypatch):
    """The same narrow networks with the plan's size threshold at zero, so that modules 4, 6 and 8
    all pool into two digits (tern_module.pool) instead of folding the window into their filters;
    odd extents in front of the pooling drop their last row and column either way."""
    from paper_1801_09449_amd import unet
    monkeypatch.setattr(unet.UNetPlan, "DIGITS_FROM_MACS", 0.0)
    check_unet(G, synth.unet_table1(seed=5, n=3, width_div=8, size=(84, 76), slices=5))
    check_unet(G, synth.unet_table1(seed=6, n=1, width_div=3, size=(92, 100), slices=15))


def test_unet_table1_full_size(G):
    """The network at the paper's size (236 x 172 x 15 stack, full channel counts), one stack."""
    check_unet(G, synth.unet_table1(seed=0, n=1))


def test_net_forward_generic_wiring(G):
    """tern_net_forward beyond the Table 1 pattern: a 3-D network with padded and strided
    modules, upsampling without a skip, a skip without upsampling, a skip of a skip, unaligned
    channel counts, and no prediction layer."""
    import torch
    from paper_1801_09449_amd import unet
    n, vol = 2, (6, 14, 12)
    x = synth.gaussian((n, 3) + vol, 91, synth.T_F32)
    in_lo = np.array([-0.4, -0.5, -0.2], np.float32)
    in_hi = np.array([0.5, 0.3, 0.6], np.float32)
    spec = [
        # c_out, c_in, k, stride, pad, extras
        (20, 3, (3, 3, 3), (1, 1, 1), (1, 1, 1), dict(save="a")),
        (33, 20, (3, 3, 3), (2, 2, 2), (1, 1, 1), dict(save="b")),
        (16, 33, (1, 1, 1), (1, 1, 1), (0, 0, 0), dict()),
        (24, 16 + 33, (3, 3, 3), (1, 1, 1), (1, 1, 1), dict(concat="b")),                 # skip, no upsampling
        (12, 24, (3, 3, 3), (1, 1, 1), (1, 1, 1), dict(up=(2, 2, 2), save="c")),           # upsampling, no skip
        (8, 12 + 20, (3, 3, 3), (1, 1, 1), (0, 0, 0), dict(concat="a")),                   # same extent as "a"
        (5, 8 + 12, (1, 3, 3), (1, 1, 1), (0, 0, 0), dict(concat="c")),                    # "c" is larger: cropped
    ]
    layers = []
    for li, (co, ci, k, st, pd, extra) in enumerate(spec, start=1):
        w = synth.ternary((co, ci) + k, 0.5, 91, synth.T_WGT + 8 * li)
        lo, hi = synth.bn_like_thresholds(co, int(np.prod(k)), ci, 0.5, 0.6, 91, synth.T_THR + 8 * li)
        layers.append(dict(w=w, k=k, stride=st, pad=pd, lo=lo, hi=hi, pool=None, up=extra.get("up"),
                           concat=extra.get("concat"), save=extra.get("save")))
    plan = unet.UNetPlan(layers, None, None, in_lo, in_hi)
    pred, kept = unet.unet_forward(plan, G.dev(x), keep_layers=True)
    torch.cuda.synchronize()
    assert pred is None
    codes, _ = oracle.unet_forward(x, in_lo, in_hi, layers, None, None)
    assert len(kept) == len(codes) == 7
    for li, ((t, c), want) in enumerate(zip(kept, codes), start=1):
        assert c == want.shape[1]
        np.testing.assert_array_equal(G.words(t), oracle.pack(want), err_msg=f"module {li}")
    assert len(np.unique(codes[-1])) == 3


def test_net_forward_one_channel_first_module(G):
    """A plain chain through tern_net_forward whose first module qualifies for the gathered-tap
    route (one input channel, 3x3x3): same codes as the oracle's chain, module by module."""
    import torch
    from paper_1801_09449_amd import unet
    f = synth.config2(seed=8, vol=(12, 20, 18))
    layers = [dict(w=L["w"], k=L["k"], stride=L["stride"], pad=L["pad"], lo=L["lo"], hi=L["hi"], pool=None,
                   up=None, concat=None, save=None) for L in f.layers]
    plan = unet.UNetPlan(layers, None, None, f.in_lo, f.in_hi)
    _, kept = unet.unet_forward(plan, G.dev(f.x), keep_layers=True)
    torch.cuda.synchronize()
    want = oracle.fcn_forward(f.x, f.in_lo, f.in_hi,
                              [dict(w=L["w"], geom=ConvGeom(L["k"], L["stride"], L["pad"], L["dil"]), lo=L["lo"],
                                    hi=L["hi"]) for L in f.layers])
    for li, ((t, c), code) in enumerate(zip(kept, want), start=1):
        np.testing.assert_array_equal(G.words(t), oracle.pack(code), err_msg=f"module {li}")
