"""GPU parity of the binary special case (Eq. 8: c - 2 popcount(I xor W)) against the CPU oracle:
tern_pack_filters_binary / tern_conv3d_binary on inputs without zeros (padded borders, strides,
dilation, ragged channel counts), on ternary inputs (the mask plane is honoured), and at the
shape of BASELINE config[1].  Integer accumulators and packed codes must match exactly."""
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


def binary_case(name, n, ci, co, vol, k=3, stride=1, pad=1, dil=1, seed=0, p0_a=0.0):
    """Weights in {-1, +1}; activations without zeros by default (p0_a = 0)."""
    return synth.conv_case(name, n, ci, co, vol, k, stride, pad, dil, p0_w=0.0, p0_a=p0_a, seed=seed)


def run_binary(G, c):
    import torch
    import paper_1801_09449_amd as T
    act = T.tern_pack(G.dev(c.act))
    bank = T.tern_pack_filters_binary(G.dev(c.wgt))
    ci, co = c.act.shape[1], c.wgt.shape[0]
    acc = T.tern_conv3d_binary(act, ci, bank, co, c.k, c.stride, c.pad, c.dil)
    packed = T.tern_conv3d_binary(act, ci, bank, co, c.k, c.stride, c.pad, c.dil,
                                  thr_lo=G.dev(c.lo), thr_hi=G.dev(c.hi))
    torch.cuda.synchronize()
    return acc.cpu().numpy(), G.words(packed)


def check_binary(G, c):
    acc, packed = run_binary(G, c)
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    assert acc.shape == want.shape
    np.testing.assert_array_equal(acc, want)
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(want, c.lo, c.hi)))
    return acc


@pytest.mark.parametrize("co,ci,k", [(32, 32, (3, 3, 3)), (5, 1, (3, 3, 3)), (33, 70, (1, 3, 2)), (64, 64, (3, 3, 3)),
                                     (40, 16, (3, 3, 3)), (16, 256, (1, 1, 1)), (7, 100, (2, 1, 3))])
def test_binary_bank_layout(G, co, ci, k):
    """[tap * nchunk + chunk][co_pad][wc] sign words, by pure re-indexing of the weights."""
    import paper_1801_09449_amd as T
    w = synth.ternary((co, ci) + k, 0.0, 401, synth.T_WGT)
    got = G.words(T.tern_pack_filters_binary(G.dev(w)))
    taps = int(np.prod(k))
    wd = (ci + 31) // 32
    wc = 2 if wd % 2 == 0 else 1
    nchunk = wd // wc
    co_pad = (co + 31) // 32 * 32
    neg = np.zeros((co, wd * 32, taps), dtype=np.uint64)
    neg[:, :ci] = (w.reshape(co, ci, taps) < 0)
    words = (neg.reshape(co, wd, 32, taps) << np.arange(32, dtype=np.uint64)[None, None, :, None]).sum(axis=2)
    want = np.zeros((taps, nchunk, co_pad, wc), dtype=np.uint32)
    want[:, :, :co] = np.transpose(words.reshape(co, nchunk, wc, taps), (3, 1, 0, 2)).astype(np.uint32)
    assert got.size * 4 == T.tern_binary_bank_bytes(co, ci, k)
    np.testing.assert_array_equal(got, want.reshape(-1))


BINARY = [
    # name, n, c_in, c_out, vol, k, stride, pad, dil
    ("c64",       1,  64,  64, (6, 10, 12),  3, 1, 1, 1),
    ("c32",       1,  32,  32, (8, 8, 8),    3, 1, 1, 1),
    ("c1",        1,   1,  16, (5, 9, 9),    3, 1, 1, 1),
    ("c3",        2,   3,   5, (5, 7, 9),    3, 1, 1, 1),
    ("c16",       1,  16,  32, (6, 8, 10),   3, 1, 1, 1),
    ("c31_co33",  1,  31,  33, (5, 9, 7),    3, 1, 1, 1),
    ("c33_co17",  1,  33,  17, (5, 8, 9),    3, 1, 1, 1),
    ("c70",       1,  70,  48, (4, 9, 10),   3, 1, 1, 1),
    ("c96",       1,  96,  40, (4, 7, 9),    3, 1, 1, 1),
    ("c128",      2, 128,  32, (4, 9, 8),    3, 1, 1, 1),
    ("c256",      1, 256,  96, (5, 6, 9),    3, 1, 1, 1),
    ("tiny_vol",  1,  32,  32, (2, 3, 2),    3, 1, 1, 1),
    ("s2_odd",    1,  32,  32, (9, 11, 13),  3, 2, 1, 1),
    ("s2_even",   2,  64,  32, (8, 12, 16),  3, 2, 1, 1),
    ("dil2",      1,  32,  16, (9, 10, 11),  3, 1, 2, 2),
    ("dil3",      1,  64,  32, (10, 9, 12),  3, 1, 3, 3),
    ("k1",        1,  64,  64, (5, 9, 11),   1, 1, 0, 1),
    ("valid",     1,  32,  32, (7, 9, 11),   3, 1, 0, 1),
    ("wide_pad",  1,  64,  16, (5, 6, 7),    3, 1, 2, 1),
    ("aniso",     1,  40,  24, (6, 11, 12), (1, 3, 2), (1, 2, 1), (0, 2, 1), (1, 2, 1)),
    ("k5_s3",     1,   8,  16, (11, 12, 13), (5, 3, 1), (3, 1, 2), (2, 1, 0), (1, 1, 1)),
    ("plane",     4,  64,  64, (1, 21, 14), (1, 3, 3), 1, (0, 1, 1), 1),
    ("batch3",    3,  32,  64, (4, 8, 8),    3, 1, 1, 1),
    ("mid",       1,  64,  64, (20, 24, 24), 3, 1, 1, 1),
]


@pytest.mark.parametrize("spec", BINARY, ids=[s[0] for s in BINARY])
def test_binary_conv_without_zeros(G, spec):
    name, n, ci, co, vol, k, s, p, d = spec
    check_binary(G, binary_case(name, n, ci, co, vol, k, s, p, d, seed=409))


def test_binary_interior_equals_eq8_closed_form(G):
    """Away from the padded border an input without zeros gives c - 2 popcount(I xor W), with
    c = k-volume x C_in, evaluated here on unpacked sign bits (not through the oracle)."""
    c = binary_case("eq8", 1, 40, 8, (6, 7, 8), seed=419)
    acc, _ = run_binary(G, c)
    sa = (c.act[0] < 0)                         # [C][D][H][W]
    sw = (c.wgt < 0)                            # [Co][C][3][3][3]
    for (z, y, x) in [(1, 1, 1), (3, 4, 5), (4, 5, 6), (2, 3, 1)]:
        patch = sa[:, z - 1:z + 2, y - 1:y + 2, x - 1:x + 2]
        for co in range(8):
            ham = int(np.count_nonzero(patch ^ sw[co]))
            assert acc[0, co, z, y, x] == 27 * 40 - 2 * ham


@pytest.mark.parametrize("spec", BINARY[:12] + BINARY[12:20:2], ids=[s[0] for s in BINARY[:12] + BINARY[12:20:2]])
def test_binary_filters_on_ternary_activations(G, spec):
    """Activations with zeros: the mask plane is honoured, so the result is still the integer
    inner product of the ternary patch with the +-1 filter."""
    name, n, ci, co, vol, k, s, p, d = spec
    check_binary(G, binary_case(name, n, ci, co, vol, k, s, p, d, seed=421, p0_a=0.4))


def test_binary_zero_weight_reads_as_plus_one_and_sign_activation(G):
    import torch
    import paper_1801_09449_amd as T
    c = binary_case("zw", 1, 64, 32, (5, 8, 9), seed=431)
    w0 = c.wgt.copy()
    w0.reshape(-1)[::7] = 0                      # not in the domain: documented to read as +1
    bank0 = T.tern_pack_filters_binary(G.dev(w0))
    bank1 = T.tern_pack_filters_binary(G.dev(np.where(w0 == 0, 1, w0).astype(np.int8)))
    assert torch.equal(bank0, bank1)
    # lo = hi + 1: no zero band, the output is a sign activation without zeros
    c.hi = synth.uniform_int(32, -6, 6, 433, synth.T_THR).astype(np.int32)
    c.lo = (c.hi + 1).astype(np.int32)
    act = T.tern_pack(G.dev(c.act))
    bank = T.tern_pack_filters_binary(G.dev(c.wgt))
    packed = G.words(T.tern_conv3d_binary(act, 64, bank, 32, thr_lo=G.dev(c.lo), thr_hi=G.dev(c.hi)))
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    code = np.where(want > c.hi[None, :, None, None, None], 1, -1).astype(np.int8)
    np.testing.assert_array_equal(packed, oracle.pack(code))
    assert (packed[..., 0, 0] == 0xFFFFFFFF).all()


def test_binary_matches_ternary_kernel_on_the_same_filters(G):
    """A +-1 filter is also a ternary filter: both kernels must give the same integers."""
    import torch
    import paper_1801_09449_amd as T
    c = binary_case("both", 2, 96, 48, (6, 9, 10), seed=439, p0_a=0.3)
    act = T.tern_pack(G.dev(c.act))
    a = T.tern_conv3d_binary(act, 96, T.tern_pack_filters_binary(G.dev(c.wgt)), 48)
    b = T.tern_conv3d(act, 96, T.tern_pack_filters(G.dev(c.wgt)), 48)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_binary_kernel_variants(G):
    """Voxels per lane, channels per pass and tap splits forced through the tuning options."""
    import paper_1801_09449_amd as T
    cases = [binary_case("v_a", 1, 64, 48, (7, 13, 11), seed=443), binary_case("v_b", 2, 32, 40, (6, 9, 10), seed=444),
             binary_case("v_c", 1, 128, 32, (5, 8, 8), stride=2, seed=445),
             binary_case("v_d", 3, 64, 64, (1, 12, 12), k=(1, 3, 3), pad=(0, 1, 1), seed=446, p0_a=0.4)]
    try:
        for depth, cb, split in [(1, 32, 0), (2, 32, 0), (1, 16, 0), (2, 16, 0), (4, 16, 0), (0, 0, 2), (0, 16, 4), (2, 32, 8)]:
            T.tern_set_option(1, depth); T.tern_set_option(3, cb); T.tern_set_option(5, split)
            for c in cases:
                check_binary(G, c)
    finally:
        T.tern_set_option(1, 0); T.tern_set_option(3, 0); T.tern_set_option(5, 0)


def test_binary_persistent_workgroups(G):
    """The persistent form of the tiled kernel on binary filters, at config[1]'s shape."""
    import paper_1801_09449_amd as T
    c = synth.conv_case("cfg1_binary", 1, 64, 64, 64, p0_w=0.0, p0_a=0.0, seed=5, thr_range=(-24, 24))
    T.tern_set_option(8, 1)
    try:
        check_binary(G, c)
        assert T.tern_last_launch()["kernel"] == T.KERNEL_PERSISTENT
    finally:
        T.tern_set_option(8, 0)


def test_binary_oversized_halo_takes_the_direct_kernel(G):
    check_binary(G, binary_case("fallback", 1, 40, 33, (20, 21, 22), k=3, stride=1, pad=60, dil=60, seed=449))


def test_binary_config1_shape_every_output(G):
    """C_in = C_out = 64 on 64^3, 3^3, stride 1, pad 1, inputs without zeros: every accumulator
    and every packed code against the oracle."""
    c = synth.conv_case("cfg1_binary", 1, 64, 64, 64, p0_w=0.0, p0_a=0.0, seed=0, thr_range=(-24, 24))
    check_binary(G, c)
