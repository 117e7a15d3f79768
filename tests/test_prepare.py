"""Host-side model preparation: the weight ternariser of Eq. 4 and the folding of scale +
batch-norm + Eq. 6 into integer cut points.  The oracle (oracle/prepare_oracle.py) is pinned to
hand-worked values and closed forms; the library's host functions are then compared with it."""
import math

import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom


@pytest.fixture(scope="module")
def T():
    import os
    import paper_1801_09449_amd as T
    if not os.path.exists(T.lib_path()):
        from paper_1801_09449_amd import build
        build.build()
    return T


# ---- pins of the oracle -----------------------------------------------------------------------
def test_oracle_ternarize_hand_worked_example():
    # sum|w| = 2.35, n = 6, Delta = 0.7 * 2.35 / 6 = 0.27416..., kept = {0.9, 0.5, 0.8}
    w = np.array([[0.9, -0.1, 0.5, -0.8, 0.05, 0.0]])
    codes, alpha = oracle.ternarize_filters(w)
    np.testing.assert_array_equal(codes, [[1, 0, 1, -1, 0, 0]])
    assert alpha[0] == pytest.approx((0.9 + 0.5 + 0.8) / 3, rel=1e-15)
    # a filter of equal magnitudes keeps everything (Delta = 0.7 v < v), alpha = v
    codes, alpha = oracle.ternarize_filters(np.array([[2.0, -2.0, 2.0, -2.0]]))
    np.testing.assert_array_equal(codes, [[1, -1, 1, -1]])
    assert alpha[0] == 2.0
    # all zeros: nothing kept, alpha 0
    codes, alpha = oracle.ternarize_filters(np.zeros((1, 5)))
    assert not codes.any() and alpha[0] == 0.0


def test_oracle_ternarize_invariants_and_gaussian_sparsity():
    w = synth.gaussian((8, 4, 3, 3, 3), 7, synth.T_F32).astype(np.float64)
    codes, alpha = oracle.ternarize_filters(w)
    c2, a2 = oracle.ternarize_filters(4.0 * w)           # exact scaling by a power of two
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_allclose(a2, 4.0 * alpha, rtol=1e-15)
    c3, a3 = oracle.ternarize_filters(-w)
    np.testing.assert_array_equal(c3, -codes)
    np.testing.assert_array_equal(a3, alpha)
    # filters are independent: row 3 alone gives the same row
    c4, a4 = oracle.ternarize_filters(w[3:4])
    np.testing.assert_array_equal(c4[0], codes[3]); assert a4[0] == alpha[3]
    # N(0,1) weights: Delta -> 0.7*sqrt(2/pi); zero fraction -> erf(Delta/sqrt 2) = 0.4235
    big = synth.gaussian((4, 1 << 16), 9, synth.T_F32).astype(np.float64)
    cb, ab = oracle.ternarize_filters(big)
    want_zero = math.erf(0.7 * math.sqrt(2 / math.pi) / math.sqrt(2))
    assert abs(np.mean(cb == 0) - want_zero) < 0.01
    # alpha = E[|w| given |w| > Delta] for a unit normal
    d = 0.7 * math.sqrt(2 / math.pi)
    want_alpha = math.sqrt(2 / math.pi) * math.exp(-d * d / 2) / (1 - math.erf(d / math.sqrt(2)))
    assert np.all(np.abs(ab - want_alpha) < 0.02)


def test_oracle_sparse_ternarize_hand_worked_and_properties():
    # magnitudes 0.9 0.1 0.5 0.8 0.5 0.0: the three smallest are 0.0, 0.1 and the first of the 0.5s
    w = np.array([[0.9, -0.1, 0.5, -0.8, -0.5, 0.0]])
    codes, alpha = oracle.ternarize_filters_sparse(w, 3)
    np.testing.assert_array_equal(codes, [[1, 0, 0, -1, -1, 0]])
    assert alpha[0] == pytest.approx((0.9 + 0.8 + 0.5) / 3, rel=1e-15)
    # nothing zeroed: plain signs (an exact zero has no sign); everything zeroed: alpha 0
    codes, alpha = oracle.ternarize_filters_sparse(w, 0)
    np.testing.assert_array_equal(codes, [[1, -1, 1, -1, -1, 0]])
    assert alpha[0] == pytest.approx(2.8 / 5, rel=1e-15)
    codes, alpha = oracle.ternarize_filters_sparse(w, 6)
    assert not codes.any() and alpha[0] == 0.0
    with pytest.raises(ValueError):
        oracle.ternarize_filters_sparse(w, 7)
    # continuous weights: exactly `zeros` zeros per filter, a threshold separates zeroed from kept
    # magnitudes, kept entries carry their sign, alpha is their mean magnitude
    g = synth.gaussian((6, 4, 3, 3, 3), 13, synth.T_F32).astype(np.float64)
    per = g[0].size
    for zeros in (0, 1, per // 2, per - 1):
        codes, alpha = oracle.ternarize_filters_sparse(g, zeros)
        flat, cf = np.abs(g).reshape(6, -1), codes.reshape(6, -1)
        assert (np.sum(cf == 0, axis=1) == zeros).all()
        for co in range(6):
            z, k = flat[co][cf[co] == 0], flat[co][cf[co] != 0]
            if z.size and k.size:
                assert z.max() <= k.min()
            np.testing.assert_array_equal(cf[co][cf[co] != 0], np.sign(g[co].reshape(-1))[cf[co] != 0])
            assert alpha[co] == pytest.approx(k.mean() if k.size else 0.0, rel=1e-14)
    # given the zero count that Eq. 4's own Delta produces, the rule reproduces Eq. 4 filter by filter
    want_c, want_a = oracle.ternarize_filters(g)
    for co in range(6):
        z = int(np.sum(want_c[co] == 0))
        c1, a1 = oracle.ternarize_filters_sparse(g[co:co + 1], z)
        np.testing.assert_array_equal(c1[0], want_c[co])
        assert a1[0] == pytest.approx(want_a[co], rel=1e-14)
    # half of N(0,1) weights zeroed: the implied Delta is the median magnitude 0.6745, and
    # alpha = E[|w| given |w| > median] = 2 * phi(0.6745) / 0.5
    big = synth.gaussian((4, 1 << 16), 9, synth.T_F32).astype(np.float64)
    cb, ab = oracle.ternarize_filters_sparse(big, 1 << 15)
    kept_min = np.array([np.abs(big[i])[cb[i] != 0].min() for i in range(4)])
    assert np.all(np.abs(kept_min - 0.6745) < 0.01)
    want_alpha = 2 * math.exp(-0.6745 ** 2 / 2) / math.sqrt(2 * math.pi) / 0.5
    assert np.all(np.abs(ab - want_alpha) < 0.01)
    # sign symmetry and exact power-of-two scaling
    c2, a2 = oracle.ternarize_filters_sparse(-4.0 * g, per // 2)
    c1, a1 = oracle.ternarize_filters_sparse(g, per // 2)
    np.testing.assert_array_equal(c2, -c1)
    np.testing.assert_allclose(a2, 4.0 * a1, rtol=1e-15)


def test_oracle_activation_code_is_eq6():
    acc = np.array([-3, -2, -1, 0, 1, 2, 3])
    # y = 0.5*acc: ties at acc = +-1 fall in the inclusive zero band
    np.testing.assert_array_equal(oracle.activation_code(acc, 0.5, 0.0), [-1, -1, 0, 0, 0, 1, 1])
    # y = acc - 1.25
    np.testing.assert_array_equal(oracle.activation_code(acc, 1.0, -1.25), [-1, -1, -1, -1, 0, 1, 1])
    # negative scale mirrors
    np.testing.assert_array_equal(oracle.activation_code(acc, -0.5, 0.0), [1, 1, 0, 0, 0, -1, -1])
    a, b = oracle.bn_affine([2.0], [3.0], [0.5], [4.0], [0.25 - 1e-5], 1e-5)
    assert a[0] == pytest.approx(2.0 * 3.0 / 0.5) and b[0] == pytest.approx(0.5 - 3.0 * 4.0 / 0.5)


# ---- library vs oracle ------------------------------------------------------------------------
def test_ternarize_filters_matches_oracle(T):
    w = synth.gaussian((16, 8, 3, 3, 3), 11, synth.T_F32)
    w[0] = 0.0
    w[1] *= 1e-3
    codes, alpha = T.tern_ternarize_filters(w)
    want_c, want_a = oracle.ternarize_filters(w)
    np.testing.assert_array_equal(codes, want_c)
    np.testing.assert_allclose(alpha, want_a, rtol=1e-12, atol=0)
    assert codes.dtype == np.int8 and codes.shape == w.shape


def test_ternarize_filters_sparse_matches_oracle(T):
    w = synth.gaussian((12, 8, 3, 3, 3), 17, synth.T_F32)
    w[0] = 0.0
    w[1, :3] = 0.25          # ties, also across the cut
    w[1, 3:6] = -0.25
    w[2] = np.round(w[2] * 4) / 4   # many equal magnitudes
    per = w[0].size
    for zeros in (0, 1, per // 2, per - 1, per):
        codes, alpha = T.tern_ternarize_filters_sparse(w, zeros)
        want_c, want_a = oracle.ternarize_filters_sparse(w, zeros)
        np.testing.assert_array_equal(codes, want_c)
        np.testing.assert_allclose(alpha, want_a, rtol=1e-12, atol=0)
    assert codes.dtype == np.int8 and codes.shape == w.shape
    with pytest.raises(Exception):
        T.tern_ternarize_filters_sparse(w, per + 1)
    with pytest.raises(Exception):
        T.tern_ternarize_filters_sparse(w, -1)


def rule(acc, lo, hi):
    return np.where(acc > hi, 1, np.where(acc < lo, -1, 0)).astype(np.int8)


@pytest.mark.parametrize("bound", [27, 216, 6912])
def test_fold_thresholds_exhaustive(T, bound):
    """For every integer accumulator in range the integer rule equals Eq. 6 in float64 (P10)."""
    n = 200
    u = synth.uniform01(4 * n, 13, 3).reshape(n, 4)
    scale = np.where(u[:, 0] < 0.1, 0.0, (u[:, 1] - 0.3) * 4.0 / math.sqrt(bound))   # some zero, some negative
    shift = (u[:, 2] - 0.5) * 3.0
    # constructed ties and saturated channels
    scale[:6] = [0.5, 0.25, -0.5, 0.0, 0.0, 0.0]
    shift[:6] = [0.0, 0.5, 0.0, 0.7, -0.6, 0.2]
    lo, hi, neg = T.tern_fold_thresholds(scale, shift, bound)
    acc = np.arange(-bound, bound + 1)
    assert np.all(lo.astype(np.int64) <= hi.astype(np.int64) + 1)
    for c in range(n):
        eff = -acc if neg[c] else acc            # accumulator the caller sees after negating the filter
        want = oracle.activation_code(eff, scale[c], shift[c])
        np.testing.assert_array_equal(rule(acc, lo[c], hi[c]), want, err_msg=f"channel {c}")
        assert neg[c] == (1 if scale[c] < 0 else 0)
    # the hand cases: y = 0.5 acc -> zero band [-1, 1]
    assert (lo[0], hi[0]) == (-1, 1)
    assert (lo[2], hi[2], neg[2]) == (-1, 1, 1)
    assert hi[3] == -bound - 1                     # constant +1
    assert lo[4] == bound + 1                      # constant -1
    assert lo[5] == -bound - 1 and hi[5] == bound + 1   # constant 0


def test_sparse_filters_leave_no_filter_words_to_skip(T):
    """The remark after Eq. 9 (half of every kernel's entries zero would halve the bit counts)
    gives no mechanism.  What a GPU kernel could skip is a filter word whose mask is all-zero,
    and only where the skip is wave-uniform: a 32-channel word of one filter at one tap, the
    64-channel chunk the kernel reads per step, or the four filters x chunk that one scalar fetch
    brings in.  Measured on Gaussian filters through the library's prescribed-sparsity quantiser:
    at 50 % zeros there is not a single all-zero word, at 90 % about 3 % of the words, 0.1 % of
    the chunks and none of the fetch groups (independent zeros: 0.9^32 = 3.4 %, 0.9^64 = 0.1 %)."""
    w = synth.gaussian((64, 64, 3, 3, 3), 0, synth.T_F32)
    per = 64 * 27
    seen = {}
    for frac in (0.5, 0.7, 0.9):
        codes, _ = T.tern_ternarize_filters_sparse(w, int(round(frac * per)))
        nz = codes != 0
        assert abs(1.0 - nz.mean() - frac) < 1e-3
        words = nz.reshape(64, 2, 32, 27).any(axis=2)                 # [filter][word][tap]
        chunks = words.any(axis=1)                                     # [filter][tap]
        groups = chunks.reshape(16, 4, 27).any(axis=1)                 # four consecutive filters
        seen[frac] = (1.0 - words.mean(), 1.0 - chunks.mean(), 1.0 - groups.mean())
    assert seen[0.5] == (0.0, 0.0, 0.0)
    assert seen[0.7][0] < 1e-3 and seen[0.7][1] == 0.0
    assert 0.02 < seen[0.9][0] < 0.05 and seen[0.9][1] < 0.005 and seen[0.9][2] == 0.0


def test_fold_rejects_bad_arguments(T):
    with pytest.raises(T.TernError):
        T.tern_fold_thresholds([np.nan], [0.0], 27)
    with pytest.raises(T.TernError):
        T.tern_fold_thresholds([1.0], [0.0], 0)
    with pytest.raises(T.TernError):
        T.tern_fold_batchnorm([1.0], [1.0], [0.0], [0.0], [-1.0], 1e-5, 27)


def test_module_chain_float_reference_equals_folded_integer_path(T):
    """Float weights -> Eq. 4 -> ternary conv (oracle) -> alpha, batch-norm, Eq. 6 in float64
    equals the integer path with folded cut points and negated filters where the scale is < 0."""
    c_in, c_out, vol = 6, 10, (5, 6, 7)
    wf = synth.gaussian((c_out, c_in, 3, 3, 3), 17, synth.T_F32)
    codes, alpha = T.tern_ternarize_filters(wf)
    act = synth.ternary((1, c_in) + vol, 0.4, 17, synth.T_ACT)
    g = ConvGeom.make()
    u = synth.uniform01(4 * c_out, 17, 5).reshape(c_out, 4)
    gamma = (u[:, 0] - 0.3) * 2.0                  # some negative
    beta = (u[:, 1] - 0.5)
    mean = (u[:, 2] - 0.5) * 4.0
    var = u[:, 3] * 9.0 + 0.1
    # float64 reference of the module
    acc = oracle.conv3d(act, codes, g)
    a, b = oracle.bn_affine(alpha, gamma, beta, mean, var, 1e-5)
    want = np.stack([oracle.activation_code(acc[:, c], a[c], b[c]) for c in range(c_out)], axis=1)
    # integer path
    lo, hi, neg = T.tern_fold_batchnorm(alpha, gamma, beta, mean, var, 1e-5, 27 * c_in)
    codes2 = codes.copy()
    codes2[neg.astype(bool)] *= -1
    got = oracle.threshold(oracle.conv3d(act, codes2, g), lo, hi)
    np.testing.assert_array_equal(got, want)
    assert neg.any() and not neg.all()


@pytest.mark.gpu
@pytest.mark.parametrize("half_zero", [False, True], ids=["eq4", "half-zero"])
def test_prepared_module_on_gpu_matches_float_reference(T, half_zero):
    import torch
    c_in, c_out, vol = 40, 48, (6, 9, 10)
    wf = synth.gaussian((c_out, c_in, 3, 3, 3), 19, synth.T_F32)
    if half_zero:   # the paper's example of a prescribed sparsity: half of every filter zero
        codes, alpha = T.tern_ternarize_filters_sparse(wf, wf[0].size // 2)
        assert (np.sum(codes.reshape(c_out, -1) == 0, axis=1) == wf[0].size // 2).all()
    else:
        codes, alpha = T.tern_ternarize_filters(wf)
    act = synth.ternary((1, c_in) + vol, 0.4, 19, synth.T_ACT)
    u = synth.uniform01(4 * c_out, 19, 5).reshape(c_out, 4)
    gamma, beta, mean, var = (u[:, 0] - 0.3) * 2.0, u[:, 1] - 0.5, (u[:, 2] - 0.5) * 8.0, u[:, 3] * 25.0 + 0.1
    lo, hi, neg = T.tern_fold_batchnorm(alpha, gamma, beta, mean, var, 1e-5, 27 * c_in)
    codes2 = codes.copy(); codes2[neg.astype(bool)] *= -1
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    out = T.tern_conv3d(T.tern_pack(dev(act)), c_in, T.tern_pack_filters(dev(codes2)), c_out,
                        thr_lo=dev(lo), thr_hi=dev(hi))
    torch.cuda.synchronize()
    acc = oracle.conv3d(act, codes, ConvGeom.make())
    a, b = oracle.bn_affine(alpha, gamma, beta, mean, var, 1e-5)
    want = np.stack([oracle.activation_code(acc[:, c], a[c], b[c]) for c in range(c_out)], axis=1)
    np.testing.assert_array_equal(out.cpu().numpy().view(np.uint32), oracle.pack(want))
