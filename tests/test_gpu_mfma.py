"""GPU parity of the matrix-core route (tern_expand_filters + tern_conv3d_mfma) against the CPU
oracle, bit-exact: integer accumulators and packed ternary codes, on the shapes the bit-count
route is tested on (every BASELINE configuration, ragged volumes, strides, dilations, channel
counts that leave partial words and odd numbers of 32-filter blocks, batches, 2-D stacks)."""
import numpy as np
import pytest

import synth
from tests.test_gpu_parity import G, SMALL, check_case, check_sampled, expect  # noqa: F401

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("spec", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes(G, spec):
    name, n, ci, co, vol, k, s, p, d = spec
    c = synth.conv_case(name, n, ci, co, vol, k, s, p, d, p0_w=0.5, p0_a=0.4, seed=61)
    check_case(G, c, mfma=True)


EXTRA = [
    # odd number of 32-filter blocks (one block per workgroup), partial last block
    synth.conv_case("m_co70", 1, 100, 70, (7, 10, 9), seed=401),
    synth.conv_case("m_co130", 1, 256, 130, (4, 8, 8), k=1, pad=0, seed=402),
    # one block, fewer than 32 filters; three input channels
    synth.conv_case("m_c3", 1, 3, 20, (9, 8, 11), seed=403),
    # stack of 2-D planes, batch in front
    synth.conv_case("m_2d", 3, 128, 64, (1, 21, 14), k=(1, 3, 3), pad=0, seed=404),
    # halo tiles that only fit with fewer waves per workgroup: stride 2 and dilation 3 in 3-D
    synth.conv_case("m_s2", 1, 64, 64, (9, 12, 10), stride=2, seed=405),
    synth.conv_case("m_d3", 1, 64, 32, (10, 9, 12), pad=3, dil=3, seed=406),
    # more halo voxels than one batch of loads per thread (5 x 5 x 5 kernel)
    synth.conv_case("m_k5", 1, 32, 32, (8, 9, 10), k=5, pad=2, seed=407),
    # several tiles along every axis with ragged ends, several channel words
    synth.conv_case("m_ragged", 2, 160, 96, (19, 13, 21), seed=408),
]


@pytest.mark.parametrize("c", EXTRA, ids=[c.name for c in EXTRA])
def test_more_shapes(G, c):
    check_case(G, c, mfma=True)


def test_byte_bank_layout(G):
    """[tap][word][block][half][filter][16 bytes], codes 0x01 / 0xff / 0x00, zero past c_out and c_in."""
    import paper_1801_09449_amd as T
    co, ci, k = 40, 70, (1, 3, 2)
    w = synth.ternary((co, ci) + k, 0.4, 77, synth.T_WGT)
    bank = T.tern_expand_filters(G.dev(w)).cpu().numpy().view(np.uint8)
    taps, wd, nblk = int(np.prod(k)), (ci + 31) // 32, (co + 31) // 32
    assert bank.size == T.tern_byte_bank_bytes(co, ci, k) == taps * wd * nblk * 1024
    want = np.zeros((taps, wd, nblk, 2, 32, 16), np.uint8)
    flat = w.reshape(co, ci, taps)
    for f in range(co):
        for c in range(ci):
            want[:, c // 32, f // 32, (c % 32) // 16, f % 32, c % 16] = flat[f, c].astype(np.uint8)
    np.testing.assert_array_equal(bank.reshape(want.shape), want)


def test_extreme_cut_points_and_empty_zero_band(G):
    c = synth.conv_case("m_cut", 1, 64, 40, (5, 9, 8), seed=409)
    i32 = np.iinfo(np.int32)
    j = np.arange(40)
    c.lo = np.where(j % 4 == 0, i32.min, np.where(j % 4 == 1, i32.max, c.lo)).astype(np.int32)
    c.hi = np.where(j % 4 == 0, i32.max, np.where(j % 4 == 1, i32.max, np.where(j % 4 == 2, i32.min, c.hi))).astype(np.int32)
    c.lo = np.minimum(c.lo, c.hi)
    c.lo[3::4] = c.hi[3::4] + 1          # empty zero band: every accumulator maps to -1 or +1
    check_case(G, c, mfma=True)


def test_config0_and_config1_full(G):
    check_case(G, synth.config0(), mfma=True)
    check_case(G, synth.config1(), mfma=True)


def test_config3_and_config4_full_size_sampled(G):
    check_sampled(G, synth.config3(), mfma=True)
    for c in synth.config4_cases():
        if c.name in ("cfg4_k3_d1_pw0.5", "cfg4_k3_d3_pw0.7", "cfg4_k1_pw0.5"):
            check_sampled(G, c, count=8000, mfma=True)


def test_oversized_halo_is_refused(G):
    """A dilation whose 8 x 8 x 2 halo tile exceeds LDS: TERN_ESHAPE, nothing launched."""
    import paper_1801_09449_amd as T
    c = synth.conv_case("m_big", 1, 32, 32, (40, 40, 40), pad=16, dil=16, seed=410)
    act = T.tern_pack(G.dev(c.act)); bank = T.tern_expand_filters(G.dev(c.wgt))
    with pytest.raises(T.TernError) as e:
        T.tern_conv3d(act, 32, bank, 32, pad=16, dil=16, mfma=True)
    assert e.value.status == -2
