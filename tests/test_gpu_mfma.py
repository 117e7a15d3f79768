"""GPU parity of the matrix-core route (tern_expand_filters + tern_conv3d_mfma) against the CPU
oracle, bit-exact: integer accumulators and packed ternary codes, on the shapes the bit-count
route is tested on (every BASELINE configuration, ragged volumes, strides, dilations, channel
counts that leave partial words and odd numbers of 32-filter blocks, batches, 2-D stacks)."""
import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom
from tests.test_gpu_parity import G, SMALL, check_case, check_sampled, expect, random_case  # noqa: F401

pytestmark = pytest.mark.gpu


KINDS = ["i8", "f4"]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("spec", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes(G, spec, kind):
    name, n, ci, co, vol, k, s, p, d = spec
    c = synth.conv_case(name, n, ci, co, vol, k, s, p, d, p0_w=0.5, p0_a=0.4, seed=61)
    check_case(G, c, mfma=kind)


EXTRA = [
    # odd number of 32-filter blocks (one block per workgroup), partial last block
    synth.conv_case("m_co70", 1, 100, 70, (7, 10, 9), seed=401),
    synth.conv_case("m_co130", 1, 256, 130, (4, 8, 8), k=1, pad=0, seed=402),
    # one block, fewer than 32 filters; three input channels
    synth.conv_case("m_c3", 1, 3, 20, (9, 8, 11), seed=403),
    # stack of 2-D planes, batch in front
    synth.conv_case("m_2d", 3, 128, 64, (1, 21, 14), k=(1, 3, 3), pad=0, seed=404),
    # a single output plane (a wave takes 8 x 16 of it), ragged in both directions; with a stride
    synth.conv_case("m_plane", 1, 64, 48, (1, 37, 21), k=(1, 3, 3), pad=(0, 1, 1), seed=412),
    synth.conv_case("m_plane_s2", 1, 96, 32, (3, 30, 19), k=(3, 3, 3), stride=(1, 2, 2), pad=(0, 1, 1), seed=413),
    # halo tiles that only fit with fewer waves per workgroup: stride 2 and dilation 3 in 3-D
    synth.conv_case("m_s2", 1, 64, 64, (9, 12, 10), stride=2, seed=405),
    synth.conv_case("m_d3", 1, 64, 32, (10, 9, 12), pad=3, dil=3, seed=406),
    # more halo voxels than one batch of loads per thread (5 x 5 x 5 kernel)
    synth.conv_case("m_k5", 1, 32, 32, (8, 9, 10), k=5, pad=2, seed=407),
    # several tiles along every axis with ragged ends, several channel words
    synth.conv_case("m_ragged", 2, 160, 96, (19, 13, 21), seed=408),
]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("c", EXTRA, ids=[c.name for c in EXTRA])
def test_more_shapes(G, c, kind):
    check_case(G, c, mfma=kind)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("i", range(32))
def test_random_geometries(G, i, kind):
    """The seeded random geometries of the bit-count route's test; a halo tile too large for LDS
    (large strides or dilations) must be refused with TERN_ESHAPE, anything else must match."""
    import paper_1801_09449_amd as T
    try:
        check_case(G, random_case(i), mfma=kind)
    except T.TernError as e:
        assert e.status == -2


WINDOWS = [(1, 2, 2), (2, 1, 2), (2, 2, 1), (1, 1, 2), (1, 3, 1), (4, 1, 1), (1, 1, 1)]


def test_random_geometries_on_pooled_digits(G):
    """Sum pooling in front of 24 random geometries (stride, padding, dilation): the window sums as
    two digits, through the bit-count kernel and through the 4-bit matrix route, against the
    oracle's convolution of the sums.  The matrix route may refuse a halo too large for LDS with
    TERN_ESHAPE (the bit-count route then takes its direct kernel); most cases must run on it."""
    import paper_1801_09449_amd as T
    ran = {False: 0, "f4": 0}
    for i in range(24):
        c = random_case(i)
        win = WINDOWS[i % len(WINDOWS)]
        n, ci = c.act.shape[:2]
        co = c.wgt.shape[0]
        vol = tuple(int(v) * f for v, f in zip(c.act.shape[2:], win))
        x = synth.ternary((n, ci) + vol, 0.35, 8100 + i, synth.T_ACT)
        pooled = np.ascontiguousarray(oracle.pool_sum(x, win))
        want_acc = oracle.conv3d(pooled, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
        want_packed = oracle.pack(oracle.threshold(want_acc, c.lo, c.hi))
        dig, c2 = T.tern_pool_digits(T.tern_pack(G.dev(x)), ci, win)
        kw = dict(k=c.k, stride=c.stride, pad=c.pad, dil=c.dil, digits=True)
        bank = T.tern_pack_filters(G.dev(T.tern_digits_weights(c.wgt)))
        mbank = T.tern_expand_filters(G.dev(c.wgt), "f4")
        for b, route in ((bank, False), (mbank, "f4")):
            try:
                acc = T.tern_conv3d(dig, c2, b, co, mfma=route, **kw)
                packed = T.tern_conv3d(dig, c2, b, co, thr_lo=G.dev(c.lo), thr_hi=G.dev(c.hi), mfma=route, **kw)
            except T.TernError as e:
                assert route and e.status == -2, (i, route)
                continue
            np.testing.assert_array_equal(acc.cpu().numpy(), want_acc, err_msg=f"case {i} route {route}")
            np.testing.assert_array_equal(G.words(packed), want_packed, err_msg=f"case {i} route {route}")
            ran[route] += 1
    assert ran[False] == 24 and ran["f4"] >= 18, ran


def test_matrix_bank_layouts(G):
    """[tap][step][block][half g][filter j][4 dwords q].  int8: step = word of 32 channels, byte b
    of dword q = channel (4 g + q) + 8 b of the word, codes 0x01 / 0xff / 0x00.  4-bit: step = pair
    of words, field i of dword q = channel 4 i + q of word g of the pair, codes 0x2 / 0xa / 0x0.
    Zero past c_out and c_in."""
    import paper_1801_09449_amd as T
    co, ci, k = 40, 70, (1, 3, 2)
    w = synth.ternary((co, ci) + k, 0.4, 77, synth.T_WGT)
    taps, nblk = int(np.prod(k)), (co + 31) // 32
    flat = w.reshape(co, ci, taps)
    bank = T.tern_expand_filters(G.dev(w), "i8").cpu().numpy().view(np.uint8)
    wd = (ci + 31) // 32
    assert bank.size == T.tern_matrix_bank_bytes(co, ci, k, "i8") == taps * wd * nblk * 1024
    want = np.zeros((taps, wd, nblk, 2, 32, 4, 4), np.uint8)            # [...][g][j][q][b]
    for f in range(co):
        for c in range(ci):
            d, b = (c % 32) % 8, (c % 32) // 8
            want[:, c // 32, f // 32, d // 4, f % 32, d % 4, b] = flat[f, c].astype(np.uint8)
    np.testing.assert_array_equal(bank.reshape(want.shape), want)
    bank4 = T.tern_expand_filters(G.dev(w), "f4").cpu().numpy().view(np.uint32)
    pairs = (ci + 63) // 64
    assert bank4.size * 4 == T.tern_matrix_bank_bytes(co, ci, k, "f4") == taps * pairs * nblk * 1024
    want4 = np.zeros((taps, pairs, nblk, 2, 32, 4), np.uint32)          # [...][g][j][q]
    code = {1: 0x2, -1: 0xA, 0: 0x0}
    for f in range(co):
        for c in range(ci):
            q, i = (c % 32) % 4, (c % 32) // 4
            vals = np.array([code[int(v)] for v in flat[f, c]], np.uint32)
            want4[:, c // 64, f // 32, (c % 64) // 32, f % 32, q] |= vals << np.uint32(4 * i)
    np.testing.assert_array_equal(bank4.reshape(want4.shape), want4)


@pytest.mark.parametrize("kind", KINDS)
def test_extreme_cut_points_and_empty_zero_band(G, kind):
    c = synth.conv_case("m_cut", 1, 64, 40, (5, 9, 8), seed=409)
    i32 = np.iinfo(np.int32)
    j = np.arange(40)
    c.lo = np.where(j % 4 == 0, i32.min, np.where(j % 4 == 1, i32.max, c.lo)).astype(np.int32)
    c.hi = np.where(j % 4 == 0, i32.max, np.where(j % 4 == 1, i32.max, np.where(j % 4 == 2, i32.min, c.hi))).astype(np.int32)
    c.lo = np.minimum(c.lo, c.hi)
    c.lo[3::4] = c.hi[3::4] + 1          # empty zero band: every accumulator maps to -1 or +1
    check_case(G, c, mfma=kind)


@pytest.mark.parametrize("kind", KINDS)
def test_cut_points_beyond_the_range_of_exact_floats(G, kind):
    """Cut points at and past +-2^24 (the 4-bit kind compares floats and clamps them there: no sum
    reaches that far, so every decision is the integer one)."""
    c = synth.conv_case("m_far", 2, 96, 33, (4, 9, 10), seed=411)
    far = np.array([2 ** 24, 2 ** 24 + 1, 2 ** 24 + 5, 2 ** 30, -(2 ** 24), -(2 ** 24) - 1, -(2 ** 24) - 7, -(2 ** 30),
                    2 ** 24 - 1, -(2 ** 24) + 1, 0], np.int64)
    c.lo = far[np.arange(33) % len(far)].astype(np.int32)
    c.hi = far[(np.arange(33) * 5 + 3) % len(far)].astype(np.int32)
    swap = c.lo > c.hi + 1                       # keep lo <= hi + 1 (the documented precondition)
    c.lo[swap], c.hi[swap] = c.hi[swap], c.lo[swap]
    check_case(G, c, mfma=kind)


@pytest.mark.parametrize("kind", KINDS)
def test_config0_and_config1_full(G, kind):
    check_case(G, synth.config0(), mfma=kind)
    check_case(G, synth.config1(), mfma=kind)


@pytest.mark.parametrize("kind", KINDS)
def test_config3_and_config4_full_size_sampled(G, kind):
    check_sampled(G, synth.config3(), mfma=kind)
    for c in synth.config4_cases():
        if c.name in ("cfg4_k3_d1_pw0.5", "cfg4_k3_d3_pw0.7", "cfg4_k1_pw0.5"):
            check_sampled(G, c, count=8000, mfma=kind)


def test_oversized_halo_is_refused(G):
    """A dilation whose 8 x 8 x 2 halo tile exceeds LDS: TERN_ESHAPE, nothing launched."""
    import paper_1801_09449_amd as T
    c = synth.conv_case("m_big", 1, 32, 32, (40, 40, 40), pad=16, dil=16, seed=410)
    act = T.tern_pack(G.dev(c.act)); bank = T.tern_expand_filters(G.dev(c.wgt), "i8")
    with pytest.raises(T.TernError) as e:
        T.tern_conv3d(act, 32, bank, 32, pad=16, dil=16, mfma="i8")
    assert e.value.status == -2
