"""The chain entry point that allocates nothing (tern_fcn_forward_static) against the entry point
it is a variant of (tern_fcn_forward) and against the oracle: two calls in a row through the C
ABI, the second on a smaller input, every layer bit for bit."""
import ctypes as C

import numpy as np
import pytest

import oracle
import synth
from oracle import ConvGeom

pytestmark = pytest.mark.gpu


def layers_of(T, dev, f):
    return [T.FcnLayer(L["w"].shape[1], L["w"].shape[0], T.tern_pack_filters(dev(L["w"])), dev(L["lo"]), dev(L["hi"]),
                       L["k"], L["stride"], L["pad"], L["dil"]) for L in f.layers]


def oracle_codes(f):
    return oracle.fcn_forward(f.x, f.in_lo, f.in_hi,
                              [dict(w=L["w"], geom=ConvGeom(L["k"], L["stride"], L["pad"], L["dil"]), lo=L["lo"],
                                    hi=L["hi"]) for L in f.layers])


def test_static_scratch_chain_matches_workspace_chain_twice_in_a_row():
    import torch
    import paper_1801_09449_amd as T
    from tests.gpu_util import dev, words
    T.lib()
    assert torch.cuda.is_available()
    # first a chain with a one-channel input (gathered first layer, strides, 5 layers), then a
    # smaller one with a three-channel input (plain Eq. 6 + pack in front): the second call finds
    # the first call's activations in the array and must not be disturbed by them
    first = synth.config2(seed=11, vol=(40, 48, 24), channels=(16, 32, 32, 64, 64), strides=(1, 2, 1, 2, 1))
    second = synth.config2(seed=12, vol=(12, 20, 9), channels=(16, 32, 48), strides=(1, 1, 2), c0=3)
    for f in (first, second):
        x, lo, hi = dev(f.x), dev(f.in_lo), dev(f.in_hi)
        layers = layers_of(T, dev, f)
        assert T.tern_fcn_workspace_bytes(x.shape, layers) <= T.tern_static_scratch_bytes()
        out_ws, views_ws = T.tern_fcn_forward(x, lo, hi, layers, return_layers=True)
        ref = [words(v).copy() for v, _ in views_ws]
        out_st, views_st = T.tern_fcn_forward(x, lo, hi, layers, return_layers=True, static_scratch=True)
        torch.cuda.synchronize()
        got = [words(v.clone()) for v, _ in views_st]
        want = oracle_codes(f)
        assert len(got) == len(ref) == len(want)
        for i, (g, r, code) in enumerate(zip(got, ref, want)):
            np.testing.assert_array_equal(g, r, err_msg=f"{f.name if hasattr(f, 'name') else ''} layer {i + 1}")
            np.testing.assert_array_equal(g, oracle.pack(code), err_msg=f"layer {i + 1} against the oracle")
        np.testing.assert_array_equal(words(out_st), words(out_ws))


def test_static_scratch_chain_refuses_what_does_not_fit():
    import torch
    import paper_1801_09449_amd as T
    from tests.gpu_util import dev
    f = synth.config2(seed=13, vol=(8, 8, 8), channels=(16, 16), strides=(1, 1))
    layers = layers_of(T, dev, f)
    # 1 x 1 x 160 x 160 x 160 floats: the gathered taps and the first layer's output need 2 x 32.8 MB
    x = torch.zeros((1, 1, 160, 160, 160), dtype=torch.float32, device="cuda")
    assert T.tern_fcn_workspace_bytes(x.shape, layers) > T.tern_static_scratch_bytes()
    with pytest.raises(T.TernError) as e:
        T.tern_fcn_forward(x, dev(f.in_lo), dev(f.in_hi), layers, static_scratch=True)
    assert e.value.status == -4
