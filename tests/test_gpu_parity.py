"""GPU parity: every entry point of the C ABI against the CPU oracle, bit-exact, on the same
seeded inputs.  Integer accumulators and ternary codes must match exactly."""
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
    T.lib()          # fail loudly if the HIP library is not built
    assert torch.cuda.is_available()
    return gpu_util


def geom_of(c):
    return ConvGeom(c.k, c.stride, c.pad, c.dil)


def expect(c):
    acc = oracle.conv3d(c.act, c.wgt, geom_of(c))
    packed = oracle.pack(oracle.threshold(acc, c.lo, c.hi))
    return acc, packed


def check_case(G, c, mfma=False):
    acc, packed = G.run_case(c, mfma=mfma)
    want_acc, want_packed = expect(c)
    assert acc.shape == want_acc.shape
    np.testing.assert_array_equal(acc, want_acc)
    assert packed.shape == want_packed.shape
    np.testing.assert_array_equal(packed, want_packed)


# ---- a1: tern_pack --------------------------------------------------------------------------
@pytest.mark.parametrize("c,vol", [(1, (3, 5, 7)), (5, (4, 4, 4)), (31, (2, 3, 8)), (32, (8, 8, 8)),
                                   (33, (5, 5, 5)), (64, (8, 12, 16)), (70, (3, 3, 3)), (256, (4, 6, 8))])
def test_pack_matches_oracle(G, c, vol):
    import paper_1801_09449_amd as T
    x = synth.ternary((2, c) + vol, 0.4, 31, synth.T_ACT)
    got = G.words(T.tern_pack(G.dev(x)))
    np.testing.assert_array_equal(got, oracle.pack(x))


def test_pack_unaligned_source_and_all_code_points(G):
    import torch
    import paper_1801_09449_amd as T
    x = np.array([1, -1, 0, 0, -1, 1, 1, 0], np.int8).reshape(1, 2, 1, 1, 4)
    got = G.words(T.tern_pack(G.dev(x)))
    np.testing.assert_array_equal(got, oracle.pack(x))
    # a source that is not 4-byte aligned takes the byte path
    big = synth.ternary((1, 40, 4, 4, 8), 0.5, 37, synth.T_ACT)
    buf = torch.zeros(big.size + 1, dtype=torch.int8, device="cuda")
    buf[1:] = G.dev(big).reshape(-1)
    got = G.words(T.tern_pack(buf[1:].view(big.shape)))
    np.testing.assert_array_equal(got, oracle.pack(big))


def tiled_ternary(c, spatial, seed, period=100003):
    """[1][c][spatial] int8 ternary tensor for the large packer cases: a seeded block of `period`
    voxels per channel (a prime, so that no power-of-two stride meets the same values) repeated
    along the voxel axis; drawing hundreds of millions of values one by one would take minutes."""
    base = synth.ternary((c, period), 0.4, seed, synth.T_ACT)
    reps = -(-spatial // period)
    return np.ascontiguousarray(np.tile(base, (1, reps))[:, :spatial]).reshape(1, c, spatial)


# Every instantiation the packer's dispatch can select (voxels per thread x words held in
# registers): 16 voxels per thread needs >= 4 194 304 voxels in multiples of 16 (int8 only); four
# voxels per thread with all words in registers needs >= 262 144 voxels when there are four or
# eight words (below that the words are split over threads).
@pytest.mark.parametrize("c,vol", [(64, (128, 128, 256)), (128, (128, 128, 256)), (96, (128, 128, 256)),
                                   (160, (64, 256, 256)), (128, (64, 64, 68)), (256, (64, 64, 68)),
                                   (96, (64, 64, 68)), (64, (64, 64, 66))])
def test_pack_large_inputs_reach_every_kernel_variant(G, c, vol):
    import paper_1801_09449_amd as T
    spatial = int(np.prod(vol))
    x = tiled_ternary(c, spatial, 53 + c).reshape((1, c) + vol)
    got = G.words(T.tern_pack(G.dev(x)))
    np.testing.assert_array_equal(got, oracle.pack(x))


# ---- a6: tern_threshold_pack ----------------------------------------------------------------
@pytest.mark.parametrize("c,vol", [(3, (3, 5, 7)), (32, (4, 4, 4)), (45, (4, 6, 8)), (64, (5, 5, 5))])
def test_threshold_pack_i32(G, c, vol):
    import paper_1801_09449_amd as T
    v = synth.uniform_int(2 * c * int(np.prod(vol)), -12, 12, 41, synth.T_ACT).astype(np.int32)
    v = v.reshape((2, c) + vol)
    lo, hi = synth.threshold_pair(c, 41)
    got = G.words(T.tern_threshold_pack(G.dev(v), G.dev(lo), G.dev(hi)))
    np.testing.assert_array_equal(got, oracle.pack(oracle.threshold(v, lo, hi)))


def test_threshold_pack_i32_extreme_cut_points(G):
    import paper_1801_09449_amd as T
    v = synth.uniform_int(4 * 16, -5, 5, 43, synth.T_ACT).astype(np.int32).reshape(1, 4, 1, 4, 4)
    i32 = np.iinfo(np.int32)
    lo = np.array([i32.min, i32.min, i32.max, 0], np.int32)
    hi = np.array([i32.max, i32.min, i32.max, 0], np.int32)
    got = G.words(T.tern_threshold_pack(G.dev(v), G.dev(lo), G.dev(hi)))
    want_code = oracle.threshold(v, lo, hi)
    assert not want_code[0, 0].any() and (want_code[0, 1] == 1).all() and (want_code[0, 2] == -1).all()
    np.testing.assert_array_equal(got, oracle.pack(want_code))


def test_threshold_pack_f32_eq6_and_ties(G):
    import paper_1801_09449_amd as T
    x = synth.gaussian((2, 3, 4, 6, 8), 47, synth.T_F32)
    x.reshape(-1)[:6] = [0.5, -0.5, np.nextafter(np.float32(0.5), np.float32(1)),
                         np.nextafter(np.float32(-0.5), np.float32(-1)), np.nan, 0.0]
    lo = np.full(3, -0.5, np.float32); hi = np.full(3, 0.5, np.float32)
    got = G.words(T.tern_threshold_pack(G.dev(x), G.dev(lo), G.dev(hi)))
    np.testing.assert_array_equal(got, oracle.pack(oracle.threshold(x, lo, hi)))


@pytest.mark.parametrize("c,vol", [(64, (64, 64, 64)), (128, (64, 64, 68)), (256, (32, 64, 136)), (96, (40, 64, 64))])
def test_threshold_pack_i32_at_full_size(G, c, vol):
    """config[1]'s accumulator tensor size (64 channels on 64^3) and the four- and eight-word
    variants above the size where words are no longer split over threads; values spread like
    accumulators (within +-40), cut points in [-8, 8]."""
    import paper_1801_09449_amd as T
    spatial = int(np.prod(vol))
    period = 100003
    base = synth.uniform_int(c * period, -40, 40, 59 + c, synth.T_ACT).astype(np.int32).reshape(c, period)
    v = np.ascontiguousarray(np.tile(base, (1, -(-spatial // period)))[:, :spatial]).reshape((1, c) + vol)
    lo, hi = synth.threshold_pair(c, 59 + c)
    got = G.words(T.tern_threshold_pack(G.dev(v), G.dev(lo), G.dev(hi)))
    np.testing.assert_array_equal(got, oracle.pack(oracle.threshold(v, lo, hi)))


@pytest.mark.parametrize("c,vol", [(64, (64, 64, 64)), (256, (32, 64, 136)), (1, (128, 128, 64))])
def test_threshold_pack_f32_at_full_size(G, c, vol):
    """The float source at config[1]'s tensor size, with eight words per plane, and at
    config[2]'s input size (one channel of 128 x 128 x 64 intensities at +-0.5, Eq. 6)."""
    import paper_1801_09449_amd as T
    spatial = int(np.prod(vol))
    period = 100003
    base = synth.gaussian((c, period), 61 + c, synth.T_F32)
    x = np.ascontiguousarray(np.tile(base, (1, -(-spatial // period)))[:, :spatial]).reshape((1, c) + vol)
    u = synth.uniform01(2 * c, 61 + c, synth.T_THR).reshape(c, 2).astype(np.float32)
    lo, hi = -0.25 - u[:, 0], 0.25 + u[:, 1]
    if c == 1:
        lo, hi = np.array([-0.5], np.float32), np.array([0.5], np.float32)
    got = G.words(T.tern_threshold_pack(G.dev(x), G.dev(lo), G.dev(hi)))
    np.testing.assert_array_equal(got, oracle.pack(oracle.threshold(x, lo, hi)))


# ---- filter bank ----------------------------------------------------------------------------
@pytest.mark.parametrize("co,ci,k", [(32, 32, (3, 3, 3)), (5, 1, (3, 3, 3)), (33, 70, (1, 3, 2)),
                                     (64, 64, (3, 3, 3)), (40, 96, (1, 1, 1)), (16, 256, (3, 3, 3))])
def test_filter_bank_layout(G, co, ci, k):
    import paper_1801_09449_amd as T
    w = synth.ternary((co, ci) + k, 0.5, 53, synth.T_WGT)
    got = G.words(T.tern_pack_filters(G.dev(w)))
    want = G.bank_layout(oracle.pack(w), co, ci)
    np.testing.assert_array_equal(got, want)


# ---- a2-a5: tern_conv3d on small shapes that span tiles and ragged tails --------------------
SMALL = [
    # name, n, c_in, c_out, vol, k, stride, pad, dil
    ("c1",        1,   1,   5, (9, 10, 11), 3, 1, 1, 1),
    ("c3",        2,   3,   7, (5, 7, 9),   3, 1, 1, 1),
    ("c16",       1,  16,  32, (8, 8, 8),   3, 1, 1, 1),
    ("c31",       1,  31,  33, (6, 9, 17),  3, 1, 1, 1),
    ("c33",       1,  33,  40, (10, 9, 8),  3, 1, 1, 1),
    ("c64",       1,  64,  64, (9, 17, 10), 3, 1, 1, 1),
    ("c96",       1,  96,  70, (5, 8, 9),   3, 1, 1, 1),
    ("c128",      2, 128,  32, (4, 9, 8),   3, 1, 1, 1),
    ("c256",      1, 256,  48, (5, 6, 9),   3, 1, 1, 1),
    ("tiny_vol",  1,  32,  32, (2, 3, 2),   3, 1, 1, 1),
    ("s2_odd",    1,  32,  32, (9, 11, 13), 3, 2, 1, 1),
    ("s2_even",   2,  16,  32, (8, 12, 16), 3, 2, 1, 1),
    ("dil2",      1,  32,  16, (9, 10, 11), 3, 1, 2, 2),
    ("dil3",      1,  64,  32, (10, 9, 12), 3, 1, 3, 3),
    ("k1",        1,  64,  64, (5, 9, 11),  1, 1, 0, 1),
    ("valid",     1,  32,  32, (7, 9, 11),  3, 1, 0, 1),
    ("aniso",     1,  40,  24, (6, 11, 12), (1, 3, 2), (1, 2, 1), (0, 2, 1), (1, 2, 1)),
    ("k5_s3",     1,   8,  16, (11, 12, 13), (5, 3, 1), (3, 1, 2), (2, 1, 0), (1, 1, 1)),
    ("batch3",    3,  32,  64, (4, 8, 8),   3, 1, 1, 1),
]


@pytest.mark.parametrize("spec", SMALL, ids=[s[0] for s in SMALL])
def test_conv_small_shapes(G, spec):
    name, n, ci, co, vol, k, s, p, d = spec
    c = synth.conv_case(name, n, ci, co, vol, k, s, p, d, p0_w=0.5, p0_a=0.4, seed=61)
    check_case(G, c)


def test_conv_no_zeros_and_all_zero_inputs(G):
    # binary special case (Eq. 8): no zeros anywhere
    c = synth.conv_case("binary", 1, 64, 32, (6, 8, 8), p0_w=0.0, p0_a=0.0, seed=67)
    check_case(G, c)
    # all-zero weights / activations give all-zero accumulators
    z = synth.conv_case("zeros", 1, 32, 32, (4, 8, 8), p0_w=1.0, p0_a=0.4, seed=67)
    acc, packed = G.run_case(z)
    assert not acc.any()
    want_acc, want_packed = expect(z)
    np.testing.assert_array_equal(packed, want_packed)


def test_conv_ignores_sign_bits_under_clear_mask(G):
    import torch
    import paper_1801_09449_amd as T
    c = synth.conv_case("noncanon", 1, 64, 32, (5, 8, 9), seed=71)
    act = T.tern_pack(G.dev(c.act))
    dirty = act.clone()
    dirty[..., 1, :] = -1          # set every sign bit, also where the mask is clear
    bank = T.tern_pack_filters(G.dev(c.wgt))
    a = T.tern_conv3d(act, 64, bank, 32)
    # a set sign under a set mask flips the value, so compare against the oracle on flipped data
    flipped = np.where(c.act != 0, -np.abs(c.act), 0).astype(np.int8)
    b = T.tern_conv3d(dirty, 64, bank, 32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a.cpu().numpy(), oracle.conv3d(c.act, c.wgt, geom_of(c)))
    np.testing.assert_array_equal(b.cpu().numpy(), oracle.conv3d(flipped, c.wgt, geom_of(c)))


def test_conv_extreme_cut_points(G):
    import paper_1801_09449_amd as T
    c = synth.conv_case("extreme", 1, 32, 32, (4, 8, 8), seed=73)
    i32 = np.iinfo(np.int32)
    c.lo = np.where(np.arange(32) % 4 == 0, i32.min, np.where(np.arange(32) % 4 == 1, i32.max, c.lo)).astype(np.int32)
    c.hi = np.where(np.arange(32) % 4 == 0, i32.max, np.where(np.arange(32) % 4 == 1, i32.max,
                    np.where(np.arange(32) % 4 == 2, i32.min, c.hi))).astype(np.int32)
    c.lo = np.minimum(c.lo, c.hi)
    c.lo[3::4] = c.hi[3::4] + 1          # empty zero band: every accumulator maps to -1 or +1
    check_case(G, c)


def test_fused_equals_unfused_and_deterministic(G):
    import torch
    import paper_1801_09449_amd as T
    c = synth.conv_case("p12", 1, 64, 64, (10, 16, 16), seed=79)
    act = T.tern_pack(G.dev(c.act)); bank = T.tern_pack_filters(G.dev(c.wgt))
    lo, hi = G.dev(c.lo), G.dev(c.hi)
    acc = T.tern_conv3d(act, 64, bank, 64)
    unfused = T.tern_threshold_pack(acc, lo, hi)
    fused1 = T.tern_conv3d(act, 64, bank, 64, thr_lo=lo, thr_hi=hi)
    fused2 = T.tern_conv3d(act, 64, bank, 64, thr_lo=lo, thr_hi=hi)
    torch.cuda.synchronize()
    assert torch.equal(fused1, unfused) and torch.equal(fused1, fused2)


VARIANTS = [
    # (lane depth, waves z, channels per pass, channels per wave, tap split)
    (0, 0, 0, 0, 0), (2, 0, 16, 16, 1), (2, 0, 32, 32, 1), (4, 0, 0, 16, 1), (2, 2, 16, 48, 1),
    (2, 4, 32, 64, 1), (2, 0, 16, 0, 2), (2, 0, 16, 0, 4), (2, 0, 32, 0, 8), (4, 0, 0, 0, 2),
    (2, 2, 16, 0, 4), (1, 0, 32, 32, 1), (1, 1, 32, 32, 1), (1, 2, 32, 64, 1), (1, 4, 32, 32, 1), (1, 0, 32, 0, 2), (1, 0, 16, 16, 1), (1, 2, 16, 32, 1), (1, 0, 16, 0, 4),
    (2, 0, 0, 0, 0),
    # eight channels per pass: byte-granular stores of the packed words
    (1, 0, 8, 0, 1), (2, 0, 8, 0, 1), (1, 0, 8, 0, 2), (2, 0, 8, 0, 4), (1, 2, 8, 16, 1), (2, 0, 8, 48, 1), (0, 0, 8, 0, 8),
]


@pytest.mark.parametrize("opts", VARIANTS, ids=["-".join(map(str, v)) for v in VARIANTS])
def test_conv_kernel_variants_agree_with_oracle(G, opts):
    """Every launch shape the tuning options can force (lane depth, stacked waves, channels per
    pass / per wave, taps split over waves) on cases with one and two words per voxel, a
    tap-packed small-C_in case and a ragged channel count."""
    import paper_1801_09449_amd as T
    cases = [
        synth.conv_case("v_c64", 1, 64, 80, (6, 17, 9), seed=101),
        synth.conv_case("v_c32", 2, 32, 33, (5, 9, 10), stride=2, seed=102),
        synth.conv_case("v_c16", 1, 16, 48, (7, 9, 12), seed=103),
        synth.conv_case("v_c3_dil", 1, 3, 20, (9, 8, 11), pad=2, dil=2, seed=104),
        synth.conv_case("v_c256", 1, 256, 32, (4, 8, 8), seed=105),
    ]
    try:
        for key, val in zip((1, 2, 3, 4, 5), opts):
            T.tern_set_option(key, val)
        for c in cases:
            check_case(G, c)
    finally:
        for key in (1, 2, 3, 4, 5):
            T.tern_set_option(key, 0)


LANE_TILES = [-1, 804, 408, 404, 802, 208, 402, 204, 202, 801, 108, 104, 401]


@pytest.mark.parametrize("tile", LANE_TILES, ids=[str(v) for v in LANE_TILES])
@pytest.mark.parametrize("depth", [0, 2], ids=["auto", "v2"])
def test_wave_shapes_agree_with_oracle(G, tile, depth):
    """Every block of 64 output voxels a wave can be given (X x Y lanes in 64 / (X * Y) planes),
    on 3-D convolutions, on stacks of independent planes (kernel depth 1, batch collapsed into
    planes; extents that leave ragged tiles in x, y and z), with one and two voxels per lane, a
    tap-packed case, a single-tap case, split taps and int32 output."""
    import paper_1801_09449_amd as T
    cases = [
        synth.conv_case("w_3d", 1, 64, 48, (7, 13, 11), seed=301),
        synth.conv_case("w_3d_s2", 2, 96, 32, (9, 12, 10), stride=2, seed=302),
        synth.conv_case("w_stack", 5, 64, 64, (1, 21, 14), k=(1, 3, 3), pad=0, seed=303),
        synth.conv_case("w_stack_c32", 3, 32, 40, (2, 11, 19), k=(1, 3, 3), pad=(0, 1, 1), seed=304),
        synth.conv_case("w_stack_c512", 7, 512, 32, (1, 8, 9), k=(1, 3, 3), pad=0, seed=305),
        synth.conv_case("w_stack_tp", 4, 8, 16, (1, 12, 12), k=(1, 3, 3), pad=(0, 1, 1), seed=306),
        synth.conv_case("w_dil", 1, 64, 16, (6, 10, 10), pad=2, dil=2, seed=307),
        # a single tap kept in the tiled kernel: halo tiles one voxel wide for X = 1
        synth.conv_case("w_k1", 3, 128, 40, (3, 5, 5), k=1, pad=0, seed=308),
    ]
    try:
        T.tern_set_option(7, tile)
        T.tern_set_option(1, depth)
        T.tern_set_option(6, 0)
        for c in cases:
            check_case(G, c)
    finally:
        T.tern_set_option(7, 0)
        T.tern_set_option(1, 0)
        T.tern_set_option(6, 1)


def random_case(i):
    """Seeded random geometry: channels up to 300, extents up to 20, kernels up to 5 per axis with
    random stride, padding and dilation (kept valid), batch up to 3."""
    u = synth.uniform_int(16, 0, 10 ** 6, 9000 + i, 11)
    pick = lambda j, lo, hi: int(lo + u[j] % (hi - lo + 1))
    c_in = [1, 3, 8, 16, 17, 32, 33, 64, 65, 100, 128, 200, 256, 300][pick(0, 0, 13)]
    c_out = [1, 5, 16, 17, 31, 32, 33, 48, 64, 70, 96, 129][pick(1, 0, 11)]
    n = pick(2, 1, 3)
    k = tuple(pick(3 + a, 1, 5 if c_in <= 64 else 3) for a in range(3))
    dil = tuple(pick(6 + a, 1, 3) for a in range(3))
    stride = tuple(pick(9 + a, 1, 3) for a in range(3))
    pad = tuple(pick(12 + a, 0, dil[a] * (k[a] - 1)) for a in range(3))
    vol = tuple(max(dil[a] * (k[a] - 1) + 1 - 2 * pad[a], 1) + pick(15, 0, 12) + 3 * a for a in range(3))
    return synth.conv_case(f"rnd{i}", n, c_in, c_out, vol, k, stride, pad, dil, seed=7000 + i)


@pytest.mark.parametrize("i", range(48))
def test_random_geometries(G, i):
    check_case(G, random_case(i))


def test_generic_fallback_for_oversized_halo(G):
    # dilation so large that no halo tile fits in LDS: the library falls back to the direct kernel
    c = synth.conv_case("fallback", 1, 40, 33, (20, 21, 22), k=3, stride=1, pad=60, dil=60, seed=83)
    check_case(G, c)
    c2 = synth.conv_case("fallback2", 1, 8, 8, (70, 9, 9), k=(2, 1, 1), stride=1, pad=(0, 0, 0),
                         dil=(64, 1, 1), seed=83)
    check_case(G, c2)


# ---- BASELINE configurations -----------------------------------------------------------------
def test_config0_full(G):
    check_case(G, synth.config0())


def test_config1_full(G):
    check_case(G, synth.config1())


def sample_points(shape, count, seed):
    n, co, d, h, w = shape
    u = synth.uniform01(5 * count, seed, 9).reshape(count, 5)
    pts = np.floor(u * np.array([n, co, d, h, w])).astype(np.int32)
    # always include the corners and the last element
    extra = np.array([[0, 0, 0, 0, 0], [n - 1, co - 1, d - 1, h - 1, w - 1], [0, co - 1, 0, h - 1, 0],
                      [n - 1, 0, d - 1, 0, w - 1]], np.int32)
    return np.concatenate([pts, extra])


def check_sampled(G, c, count=20000, mfma=False):
    """Full-size run; the oracle computes a random sample of outputs one by one."""
    acc, packed = G.run_case(c, mfma=mfma)
    pts = sample_points(acc.shape, count, 97)
    want = oracle.conv3d_points(c.act, c.wgt, geom_of(c), pts)
    got = acc[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3], pts[:, 4]]
    np.testing.assert_array_equal(got, want)
    # codes at the same points, decoded from the packed words
    co = pts[:, 1]
    mw = packed[pts[:, 0], pts[:, 2], pts[:, 3], pts[:, 4], 0, co // 32]
    sw = packed[pts[:, 0], pts[:, 2], pts[:, 3], pts[:, 4], 1, co // 32]
    m = (mw >> (co % 32).astype(np.uint32)) & 1
    s = (sw >> (co % 32).astype(np.uint32)) & 1
    code = m.astype(np.int8) * (1 - 2 * s.astype(np.int8))
    want_code = np.where(want > c.hi[co], 1, np.where(want < c.lo[co], -1, 0))
    np.testing.assert_array_equal(code, want_code)
    # properties that hold everywhere: canonical packing, bounded accumulators
    assert not (packed[..., 1, :] & ~packed[..., 0, :]).any()
    bound = c.act.shape[1] * int(np.prod(c.k))
    assert np.abs(acc).max() <= bound
    # and the fused output equals thresholding the accumulator tensor everywhere
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(acc, c.lo, c.hi)))


def test_config3_reduced_full_and_full_size_sampled(G):
    check_case(G, synth.config3(vol=(6, 9, 10), n=2))
    check_sampled(G, synth.config3())


def test_config3_full_size_every_output(G):
    """All 33.5 M accumulators and codes of config[3] against the oracle (116 GMAC of scalar
    work on the host cores: some tens of seconds)."""
    check_case(G, synth.config3())


def test_config4_reduced_full(G):
    for c in synth.config4_cases(vol=(12, 13, 20)):
        check_case(G, c)


def test_config4_full_size_sampled(G):
    """All twelve cases of the sweep at 96^3 (the oracle evaluates the sampled outputs only)."""
    cases = synth.config4_cases()
    assert len(cases) == 12
    for c in cases:
        check_sampled(G, c, count=8000)


def test_config4_pointwise_full_size_every_output(G):
    """The 1^3 case at 96^3 element by element (3.6 GMAC for the oracle)."""
    c = [c for c in synth.config4_cases() if c.name == "cfg4_k1_pw0.5"][0]
    check_case(G, c)


def fcn_run(G, f):
    import paper_1801_09449_amd as T
    layers = []
    for L in f.layers:
        layers.append(T.FcnLayer(c_in=L["w"].shape[1], c_out=L["w"].shape[0],
                                 w_bank=T.tern_pack_filters(G.dev(L["w"])),
                                 thr_lo=G.dev(L["lo"]), thr_hi=G.dev(L["hi"]),
                                 k=L["k"], stride=L["stride"], pad=L["pad"], dil=L["dil"]))
    out, views = T.tern_fcn_forward(G.dev(f.x), G.dev(f.in_lo), G.dev(f.in_hi), layers, return_layers=True)
    import torch
    torch.cuda.synchronize()
    return [(G.words(v), dm) for v, dm in views]


def fcn_expect(f):
    layers = [dict(w=L["w"], geom=ConvGeom(L["k"], L["stride"], L["pad"], L["dil"]), lo=L["lo"], hi=L["hi"])
              for L in f.layers]
    return oracle.fcn_forward(f.x, f.in_lo, f.in_hi, layers)


def test_config2_fcn_reduced(G):
    f = synth.config2(seed=3, vol=(16, 24, 16))
    got = fcn_run(G, f)
    want = fcn_expect(f)
    assert len(got) == 6
    for (w, dm), code in zip(got, want):
        assert tuple(dm) == code.shape
        np.testing.assert_array_equal(w, oracle.pack(code))
    assert got[-1][1] == (1, 128, 2, 3, 2)


def test_config2_fcn_full(G):
    f = synth.config2()
    got = fcn_run(G, f)
    want = fcn_expect(f)
    for i, ((w, dm), code) in enumerate(zip(got, want)):
        assert tuple(dm) == code.shape, f"layer {i + 1}"
        np.testing.assert_array_equal(w, oracle.pack(code), err_msg=f"layer {i + 1}")
    assert got[-1][1] == (1, 128, 16, 16, 8)
    # the synthetic cut points keep the activations from collapsing
    zero_frac = float(np.mean(want[-1] == 0))
    assert 0.15 < zero_frac < 0.7


POINTWISE = [(27, 16, (5, 7, 9), 1), (64, 64, (6, 5, 7), 2), (128, 40, (3, 5, 5), 3), (256, 96, (4, 4, 4), 1),
             (32, 33, (1, 1, 130), 2), (100, 70, (2, 9, 8), 2), (8, 200, (3, 3, 3), 1), (1, 1, (1, 1, 1), 1),
             (64, 32, (16, 32, 40), 1), (135, 32, (3, 10, 13), 2), (160, 48, (2, 7, 9), 1), (80, 64, (5, 6, 7), 1),
             (96, 17, (1, 3, 50), 3)]


@pytest.mark.parametrize("ci,co,vol,n", POINTWISE, ids=[f"{a}-{b}-n{d}" for a, b, _, d in POINTWISE])
def test_pointwise_kernel_and_tiled_route_agree_with_oracle(G, ci, co, vol, n):
    """1x1x1 convolutions: 1, 2, 3, 4, 5 and 8 input words per plane, ragged voxel counts and channel
    tails, batches; once through the pointwise kernel and once forced through the tiled one."""
    import paper_1801_09449_amd as T
    c = synth.conv_case("pw", n, ci, co, vol, k=1, pad=0, seed=ci + co)
    want_acc, want_packed = expect(c)
    try:
        for use_point in (1, 0):
            T.tern_set_option(6, use_point)
            acc, packed = G.run_case(c)
            np.testing.assert_array_equal(acc, want_acc)
            np.testing.assert_array_equal(packed, want_packed)
    finally:
        T.tern_set_option(6, 1)


FIRST_LAYERS = [
    # (k, stride, pad, dil) of layer 0 on a one-channel input; 3x3x3 and 1x3x3 kernels with unit
    # depth stride and dilation take the route that gathers the taps into one word per output
    # voxel (rows 0, 1, 3), 15x3x3 kernels the same route with five words (rows 9, 10), the others
    # the ordinary one
    ((3, 3, 3), (1, 1, 1), (1, 1, 1), (1, 1, 1)),
    ((1, 3, 3), (1, 1, 1), (0, 1, 1), (1, 1, 1)),
    ((2, 3, 3), (1, 2, 1), (1, 0, 1), (1, 1, 1)),
    ((3, 3, 3), (1, 2, 2), (1, 2, 1), (1, 2, 1)),
    ((2, 4, 4), (1, 1, 3), (0, 2, 0), (1, 1, 2)),      # 32 taps: the word is full
    ((3, 1, 5), (1, 1, 1), (2, 0, 3), (1, 1, 1)),
    ((3, 3, 3), (2, 1, 1), (1, 1, 1), (1, 1, 1)),      # depth stride 2
    ((3, 3, 3), (1, 1, 1), (2, 1, 1), (2, 1, 1)),      # depth dilation 2
    ((3, 3, 4), (1, 1, 1), (1, 1, 1), (1, 1, 1)),      # 36 taps
    ((15, 3, 3), (1, 1, 1), (2, 1, 1), (1, 1, 1)),     # stack kernel: 135 taps in five words, one output plane
    ((15, 3, 3), (1, 2, 1), (4, 0, 1), (1, 1, 1)),     # the same with five output planes
]


@pytest.mark.parametrize("k,stride,pad,dil", FIRST_LAYERS, ids=[str(i) for i in range(len(FIRST_LAYERS))])
def test_fcn_first_layer_geometries(G, k, stride, pad, dil):
    """One-channel float input, asymmetric input cut points, batch of 2, extents that are not
    multiples of the kernels' block shapes; three layers so that layer 0's output feeds on."""
    vol = (11, 70, 67)
    x = synth.gaussian((2, 1) + vol, 61, synth.T_F32)
    in_lo, in_hi = np.array([-0.3], np.float32), np.array([0.8], np.float32)
    layers, c_in = [], 1
    for li, (c_out, kk, st, pd, dl) in enumerate([(20, k, stride, pad, dil), (33, (3, 3, 3), (1, 1, 1), (1, 1, 1), (1, 1, 1)),
                                                   (8, (1, 1, 1), (1, 1, 1), (0, 0, 0), (1, 1, 1))], start=1):
        w = synth.ternary((c_out, c_in) + kk, 0.5, 61, synth.T_WGT + 8 * li)
        lo, hi = synth.bn_like_thresholds(c_out, int(np.prod(kk)), c_in, 0.5, 0.6, 61, synth.T_THR + 8 * li)
        layers.append(dict(w=w, k=kk, stride=st, pad=pd, dil=dl, lo=lo, hi=hi))
        c_in = c_out
    f = synth.FcnCase("first", x, in_lo, in_hi, layers)
    got = fcn_run(G, f)
    want = fcn_expect(f)
    for i, ((w, dm), code) in enumerate(zip(got, want)):
        assert tuple(dm) == code.shape, f"layer {i + 1}"
        np.testing.assert_array_equal(w, oracle.pack(code), err_msg=f"layer {i + 1}")
    assert len(np.unique(want[0])) == 3


@pytest.mark.parametrize("k,pad,c_out", [((3, 3, 3), (1, 1, 1), 70), ((15, 3, 3), (0, 1, 0), 33),
                                         ((1, 3, 3), (0, 0, 2), 97)], ids=["3x3x3-70", "15x3x3-33", "1x3x3-97"])
def test_fcn_first_layer_more_than_one_output_word(G, k, pad, c_out):
    """The fused first-layer kernel with more than 32 output channels (several packed words per
    voxel, a ragged last pass), followed by a layer that reads them."""
    vol = (17, 21, 70)
    x = synth.gaussian((1, 1) + vol, 67, synth.T_F32)
    in_lo, in_hi = np.array([-0.4], np.float32), np.array([0.4], np.float32)
    layers, c_in = [], 1
    for li, (co, kk, pd) in enumerate([(c_out, k, pad), (16, (1, 1, 1), (0, 0, 0))], start=1):
        w = synth.ternary((co, c_in) + kk, 0.5, 67, synth.T_WGT + 8 * li)
        lo, hi = synth.bn_like_thresholds(co, int(np.prod(kk)), c_in, 0.5, 0.6, 67, synth.T_THR + 8 * li)
        layers.append(dict(w=w, k=kk, stride=(1, 1, 1), pad=pd, dil=(1, 1, 1), lo=lo, hi=hi))
        c_in = co
    f = synth.FcnCase("first-wide", x, in_lo, in_hi, layers)
    got = fcn_run(G, f)
    want = fcn_expect(f)
    for i, ((w, dm), code) in enumerate(zip(got, want)):
        assert tuple(dm) == code.shape, f"layer {i + 1}"
        np.testing.assert_array_equal(w, oracle.pack(code), err_msg=f"layer {i + 1}")


# ---- tensors above 4 GiB: byte offsets need 64 bits, voxel indices still fit 32 ---------------
@pytest.mark.parametrize("c_in,c_out", [(1, 33), (17, 8)], ids=["tap-packed", "plain"])
def test_volume_above_4gib_sampled(G, c_in, c_out):
    """576 Mi voxels: the packed input (4.5 GiB) and output (4.5 or 9 GiB) exceed 32-bit byte
    offsets.  The volume is one seeded 64 Mi-voxel block repeated nine times along D (drawing
    every element separately would take minutes); the oracle evaluates sampled outputs, which
    include the last voxel, on the very same array."""
    import torch
    import paper_1801_09449_amd as T
    block = synth.ternary((1, c_in, 64, 1024, 1024), 1.0 / 3.0, 41, synth.T_ACT)
    act = np.tile(block, (1, 1, 9, 1, 1))
    del block
    wgt = synth.ternary((c_out, c_in, 3, 3, 3), 0.5, 41, synth.T_WGT)
    lo, hi = synth.threshold_pair(c_out, 41, lo=-2, hi=2)
    packed_in = T.tern_pack(G.dev(act))
    assert packed_in.numel() * 4 > 2 ** 32
    out = T.tern_conv3d(packed_in, c_in, T.tern_pack_filters(G.dev(wgt)), c_out, 3, 1, 1, 1,
                        thr_lo=G.dev(lo), thr_hi=G.dev(hi))
    torch.cuda.synchronize()
    del packed_in
    assert out.numel() * 4 > 2 ** 32
    pts = sample_points((1, c_out) + act.shape[2:], 3000, 43)
    pts = np.concatenate([pts, pts[:200] * np.array([0, 1, 0, 1, 1]) + np.array([0, 0, 575, 0, 0])]
                         ).astype(np.int32)                      # and the last plane
    want = oracle.conv3d_points(act, wgt, ConvGeom((3,) * 3, (1,) * 3, (1,) * 3, (1,) * 3), pts)
    idx = [torch.from_numpy(pts[:, a].astype(np.int64)).cuda() for a in (0, 2, 3, 4)]
    co = pts[:, 1]
    wsel = torch.from_numpy((co // 32).astype(np.int64)).cuda()
    mw = out[idx[0], idx[1], idx[2], idx[3], 0, wsel].cpu().numpy().view(np.uint32)
    sw = out[idx[0], idx[1], idx[2], idx[3], 1, wsel].cpu().numpy().view(np.uint32)
    m = (mw >> (co % 32).astype(np.uint32)) & 1
    s = (sw >> (co % 32).astype(np.uint32)) & 1
    code = m.astype(np.int8) * (1 - 2 * s.astype(np.int8))
    want_code = np.where(want > hi[co], 1, np.where(want < lo[co], -1, 0))
    np.testing.assert_array_equal(code, want_code)
    assert len(np.unique(want_code)) == 3
    # canonical packing everywhere, no bits above the channel count (checked on the device)
    assert not bool((out[..., 1, :] & ~out[..., 0, :]).any())
    if c_out % 32:
        assert not bool((out[..., 0, -1] >> (c_out % 32)).any())


def test_calls_follow_the_callers_stream(G):
    """Every entry point enqueues on the stream it is given: a chain issued on a side stream,
    with no synchronisation between the calls, gives the oracle's result, and work on the default
    stream in between does not disturb it."""
    import torch
    import paper_1801_09449_amd as T
    c = synth.conv_case("stream", 1, 40, 24, (10, 18, 20), seed=77)
    want_acc, want_packed = expect(c)
    side = torch.cuda.Stream()
    act8, wgt8, lo, hi = G.dev(c.act), G.dev(c.wgt), G.dev(c.lo), G.dev(c.hi)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        a = T.tern_pack(act8)
        b = T.tern_pack_filters(wgt8)
        acc = T.tern_conv3d(a, 40, b, 24, c.k, c.stride, c.pad, c.dil)
        fused = T.tern_conv3d(a, 40, b, 24, c.k, c.stride, c.pad, c.dil, thr_lo=lo, thr_hi=hi)
        two_step = T.tern_threshold_pack(acc, lo, hi)
    noise = torch.zeros(1 << 20, device="cuda").add_(1.0)      # default stream, unrelated
    side.synchronize()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), want_acc)
    np.testing.assert_array_equal(G.words(fused), want_packed)
    np.testing.assert_array_equal(G.words(two_step), want_packed)
    assert float(noise.sum()) == float(1 << 20)


def test_fcn_forward_replays_from_a_captured_graph(G):
    """The entry points allocate nothing and clear nothing, so a chain of them can be recorded
    into a HIP graph: capture tern_fcn_forward once, then replay it on new input contents, with
    eager work and synchronisation between the replays; every replay must match the oracle."""
    import torch
    import paper_1801_09449_amd as T
    f = synth.config2(seed=5, vol=(16, 24, 16))
    layers = [T.FcnLayer(c_in=L["w"].shape[1], c_out=L["w"].shape[0], w_bank=T.tern_pack_filters(G.dev(L["w"])),
                         thr_lo=G.dev(L["lo"]), thr_hi=G.dev(L["hi"]), k=L["k"], stride=L["stride"],
                         pad=L["pad"], dil=L["dil"]) for L in f.layers]
    x = G.dev(f.x)
    ilo, ihi = G.dev(f.in_lo), G.dev(f.in_hi)
    ws = torch.empty((T.tern_fcn_workspace_bytes(x.shape, layers),), dtype=torch.uint8, device="cuda")
    out = T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws)      # warm-up, also sizes `out`
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws, out=out)
    want_layers = [dict(w=L["w"], geom=ConvGeom(L["k"], L["stride"], L["pad"], L["dil"]), lo=L["lo"], hi=L["hi"])
                   for L in f.layers]
    for rep in range(3):
        xi = synth.gaussian(f.x.shape, 100 + rep, synth.T_F32)
        x.copy_(torch.from_numpy(xi))
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle.fcn_forward(xi, f.in_lo, f.in_hi, want_layers)[-1]
        np.testing.assert_array_equal(G.words(out), oracle.pack(want), err_msg=f"replay {rep}")
        # eager call on the same input gives the same bits
        eager = T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(G.words(eager), G.words(out))


@pytest.mark.gpu
def test_instruction_mix_probe_runs_every_variant(G):
    """The diagnostic kernels (no counterpart in the paper) launch in every variant and leave
    their sink alone."""
    import torch
    import paper_1801_09449_amd as T
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for variant in range(17):
        T.tern_probe_valu(64, 256, 50, sink, variant)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
