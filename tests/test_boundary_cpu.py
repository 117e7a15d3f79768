"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects invalid arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    import paper_1801_09449_amd as T
    if not os.path.exists(T.lib_path()):
        from paper_1801_09449_amd import build
        build.build()
    return T


def test_every_declared_symbol_is_exported(T):
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["tern.h", "tern_matrix.h", "tern_tuning.h"]
    names = set()
    for h in headers:
        hdr = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(tern_[a-z0-9_]+)\s*\(", hdr))
    assert {"tern_pack", "tern_conv3d", "tern_threshold_pack", "tern_fcn_forward",
            "tern_pack_filters", "tern_fcn_forward_static", "tern_conv3d_mfma", "tern_set_option"} <= names
    L = T.lib()
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in tern.h but not exported"


def test_size_helpers(T):
    assert T.tern_words(1) == 1 and T.tern_words(32) == 1 and T.tern_words(33) == 2
    assert T.tern_words(0) == 0
    assert T.tern_packed_bytes((1, 64, 64, 64, 64)) == 64 ** 3 * 16
    assert T.tern_packed_bytes((2, 1, 3, 4, 5)) == 2 * 60 * 8
    assert T.tern_packed_bytes((1, 0, 3, 4, 5)) == 0
    # filter bank: taps * words * co_pad * 8 bytes
    assert T.tern_filter_bank_bytes(64, 64, 3) == 27 * 2 * 64 * 8
    assert T.tern_filter_bank_bytes(33, 1, (1, 3, 2)) == 1 * 64 * 8      # 6 taps packed into one word
    assert T.tern_filter_bank_bytes(32, 16, 3) == 14 * 32 * 8           # two taps per word
    assert T.tern_filter_bank_bytes(32, 17, 3) == 27 * 32 * 8           # plain layout above 16 channels
    assert T.tern_filter_bank_bytes(32, 8, 1) == 1 * 32 * 8             # single tap: plain
    assert T.tern_filter_bank_bytes(0, 4, 3) == 0


def test_out_dims_formula(T):
    assert T.tern_conv_out_dims((1, 64, 64, 64, 64), 64) == (1, 64, 64, 64, 64)
    assert T.tern_conv_out_dims((1, 16, 128, 128, 64), 32, 3, 2, 1, 1) == (1, 32, 64, 64, 32)
    assert T.tern_conv_out_dims((2, 3, 7, 9, 5), 4, 3, 2, 1, 1) == (2, 4, 4, 5, 3)
    assert T.tern_conv_out_dims((1, 8, 96, 96, 96), 8, 3, 1, 3, 3) == (1, 8, 96, 96, 96)
    assert T.tern_conv_out_dims((1, 8, 9, 9, 9), 8, 1, 1, 0, 1) == (1, 8, 9, 9, 9)
    with pytest.raises(T.TernError) as e:
        T.tern_conv_out_dims((1, 8, 2, 2, 2), 8, 3, 1, 0, 1)      # kernel does not fit
    assert e.value.status == -2
    with pytest.raises(T.TernError) as e:
        T.tern_conv_out_dims((1, 8, 8, 8, 8), 8, 3, 0, 1, 1)      # stride 0
    assert e.value.status == -3


def test_null_and_bad_arguments_are_rejected_before_launch(T):
    from paper_1801_09449_amd.binding import Dims, Geom, Layer, _geom
    L = T.lib()
    d = Dims(1, 32, 4, 4, 4)
    g = _geom(3, 1, 1, 1)
    fake = C.c_void_p(0x1000)   # never dereferenced: validation fails first
    assert L.tern_pack(None, d, fake, None) == -1
    assert L.tern_pack(fake, d, None, None) == -1
    assert L.tern_pack(fake, Dims(1, 0, 4, 4, 4), fake, None) == -2
    assert L.tern_pack(fake, d, C.c_void_p(0x1004), None) == -3            # misaligned
    assert L.tern_pack_filters(None, 4, 4, 3, 3, 3, fake, None) == -1
    assert L.tern_pack_filters(fake, 4, 4, 0, 3, 3, fake, None) == -2
    assert L.tern_threshold_pack(fake, 0, d, fake, fake, fake, None) == -3  # int8 source not accepted
    assert L.tern_threshold_pack(fake, 1, d, None, fake, fake, None) == -1
    # matrix-core route: same checks as tern_pack_filters / tern_conv3d
    assert L.tern_expand_filters(None, 4, 4, 3, 3, 3, 0, fake, None) == -1
    assert L.tern_expand_filters(fake, 4, 4, 0, 3, 3, 0, fake, None) == -2
    assert L.tern_expand_filters(fake, 4, 4, 3, 3, 3, 2, fake, None) == -3                  # unknown kind
    assert L.tern_expand_filters(fake, 4, 4, 3, 3, 3, 1, C.c_void_p(0x1004), None) == -3
    assert L.tern_matrix_bank_bytes(40, 70, 1, 3, 2, 0) == 6 * 3 * 2 * 1024
    assert L.tern_matrix_bank_bytes(40, 70, 1, 3, 2, 1) == 6 * 2 * 2 * 1024
    assert L.tern_matrix_bank_bytes(0, 70, 1, 3, 2, 0) == 0
    assert L.tern_matrix_bank_bytes(40, 70, 1, 3, 2, 5) == 0
    assert L.tern_conv3d_mfma(None, d, fake, 0, 8, g, None, None, fake, None, None) == -1
    assert L.tern_conv3d_mfma(fake, d, fake, 7, 8, g, None, None, fake, None, None) == -3     # unknown kind
    assert L.tern_conv3d_mfma(fake, d, fake, 1, 8, g, None, None, fake, fake, None) == -3     # both outputs
    assert L.tern_conv3d_mfma(fake, d, fake, 0, 8, g, None, None, None, fake, None) == -1     # no cut points
    assert L.tern_conv3d_mfma(fake, Dims(1, 32, 4, 4, 0), fake, 0, 8, g, None, None, fake, None, None) == -2
    assert L.tern_conv3d_mfma_digits(None, Dims(1, 64, 4, 4, 4), fake, 8, g, None, None, fake, None, None) == -1
    assert L.tern_conv3d_mfma_digits(fake, d, fake, 8, g, None, None, fake, None, None) == -3     # 32 channels: no digit pairs
    assert L.tern_conv3d_mfma_digits(fake, Dims(1, 64, 4, 4, 4), fake, 8, g, None, None, fake, fake, None) == -3
    # conv: both or neither output, missing cut points, bad geometry
    assert L.tern_conv3d(fake, d, fake, 8, g, None, None, None, None, None) == -3
    assert L.tern_conv3d(fake, d, fake, 8, g, fake, fake, fake, fake, None) == -3
    assert L.tern_conv3d(fake, d, fake, 8, g, None, fake, None, fake, None) == -1
    assert L.tern_conv3d(None, d, fake, 8, g, None, None, fake, None, None) == -1
    assert L.tern_conv3d(fake, d, fake, 0, g, None, None, fake, None, None) == -2
    assert L.tern_conv3d(fake, d, fake, 8, _geom(3, 1, 1, 0), None, None, fake, None, None) == -3
    assert L.tern_conv3d(fake, d, fake, 8, _geom(9, 1, 0, 1), None, None, fake, None, None) == -2
    # binary filters (Eq. 8): same checks, own bank size
    assert L.tern_binary_bank_bytes(64, 64, 3, 3, 3) == 27 * 2 * 64 * 4
    assert L.tern_binary_bank_bytes(33, 1, 1, 3, 2) == 6 * 1 * 64 * 4        # no tap packing: one word per tap
    assert L.tern_binary_bank_bytes(0, 4, 3, 3, 3) == 0
    assert L.tern_pack_filters_binary(None, 4, 4, 3, 3, 3, fake, None) == -1
    assert L.tern_pack_filters_binary(fake, 4, 4, 0, 3, 3, fake, None) == -2
    assert L.tern_pack_filters_binary(fake, 4, 4, 3, 3, 3, C.c_void_p(0x1004), None) == -3
    assert L.tern_conv3d_binary(fake, d, fake, 8, g, None, None, None, None, None) == -3
    assert L.tern_conv3d_binary(fake, d, fake, 8, g, None, fake, None, fake, None) == -1
    assert L.tern_conv3d_binary(fake, d, None, 8, g, None, None, fake, None, None) == -1
    assert L.tern_conv3d_binary(fake, d, fake, 8, _geom(9, 1, 0, 1), None, None, fake, None, None) == -2
    # fcn: channel mismatch between layers, workspace too small
    arr = (Layer * 2)()
    arr[0] = Layer(32, 16, g, 0x1000, 0x1000, 0x1000)
    arr[1] = Layer(8, 16, g, 0x1000, 0x1000, 0x1000)
    assert L.tern_fcn_workspace_bytes(d, arr, 2) == 0
    arr[1] = Layer(16, 16, g, 0x1000, 0x1000, 0x1000)
    need = L.tern_fcn_workspace_bytes(d, arr, 2)
    assert need >= 64 * 8 + 64 * 8
    od = Dims()
    assert L.tern_fcn_forward(fake, d, fake, fake, arr, 2, fake, need - 1, fake, C.byref(od), None, None) == -4
    assert L.tern_fcn_forward(fake, d, fake, fake, arr, 0, fake, need, fake, C.byref(od), None, None) == -3
    assert L.tern_fcn_forward(fake, d, fake, fake, arr, 2, None, need, fake, C.byref(od), None, None) == -1
    # the same chain over the library's fixed scratch array: refused when it does not fit, before
    # any device is touched
    assert L.tern_static_scratch_bytes() == 32 << 20
    assert L.tern_fcn_forward_static(fake, d, fake, fake, arr, 2, None, C.byref(od), None, None) == -1
    assert L.tern_fcn_forward_static(fake, d, fake, fake, arr, 0, fake, C.byref(od), None, None) == -3
    big = Dims(1, 32, 128, 128, 160)       # 21 MB packed input + 21 MB first layer output
    assert L.tern_fcn_workspace_bytes(big, arr, 2) > L.tern_static_scratch_bytes()
    assert L.tern_fcn_forward_static(fake, big, fake, fake, arr, 2, fake, C.byref(od), None, None) == -4
    # two-digit pooling and convolution
    win = (C.c_int32 * 3)(1, 2, 2)
    assert L.tern_pool_digits(None, d, win, fake, None) == -1
    assert L.tern_pool_digits(fake, d, (C.c_int32 * 3)(2, 2, 2), fake, None) == -3
    assert L.tern_pool_digits(fake, d, (C.c_int32 * 3)(1, 0, 2), fake, None) == -3
    assert L.tern_conv3d_digits(fake, d, fake, 8, g, None, None, fake, None, None) == -3          # 32 channels: no digit pairs
    assert L.tern_conv3d_digits(fake, Dims(1, 64, 4, 4, 4), None, 8, g, None, None, fake, None, None) == -1
    assert L.tern_digits_weights(None, 4, 4, 27, None) == -1
    # probe: null sink, launch shape and variant are checked before anything is launched
    assert L.tern_probe_valu(4, 256, 10, 0, None, None) == -1
    assert L.tern_probe_valu(4, 100, 10, 0, fake, None) == -3
    assert L.tern_probe_valu(4, 256, 10, 17, fake, None) == -3
    assert L.tern_probe_valu(4, 256, 10, -1, fake, None) == -3
    assert L.tern_probe_valu(0, 256, 10, 1, fake, None) == -3
    # options: unknown option or value
    assert L.tern_set_option(99, 0) == -3
    assert L.tern_set_option(3, 24) == -3
    assert L.tern_set_option(3, 0) == 0
    assert L.tern_set_option(8, 2) == -3 and L.tern_set_option(8, 1) == 0 and L.tern_set_option(8, 0) == 0
    # plan query: nothing launched by this thread yet
    info = (C.c_int32 * 8)()
    assert L.tern_last_launch(None) == -1
    assert L.tern_last_launch(info) == 0 and info[0] == -1
    for bad in (1, 303, 101, 102, 1608, 816, -2):      # wave shapes: powers of two up to 8, at least 4 lanes per plane
        assert L.tern_set_option(7, bad) == -3
    for good in (808, 408, 202, 401, -1, 0):
        assert L.tern_set_option(7, good) == 0
    assert b"TERN_ESHAPE" in L.tern_status_string(-2)


def test_binding_refuses_cpu_tensors(T):
    import torch
    with pytest.raises(ValueError):
        T.tern_pack(torch.zeros((1, 4, 2, 2, 2), dtype=torch.int8))


def test_maximum_sizes_are_enforced(T):
    """The kernels index voxels with 32-bit integers and accumulate in int32: extents beyond
    those limits must be refused, extents just inside accepted (no launch: helpers only)."""
    from paper_1801_09449_amd.binding import Dims, _geom
    L = T.lib()
    fake = C.c_void_p(0x1000)
    # 2^31 - 1 voxels is the most a tensor may hold
    assert T.tern_packed_bytes((1, 1, 1, 1, 2 ** 31 - 1)) == (2 ** 31 - 1) * 8
    assert T.tern_packed_bytes((1, 1, 2, 2 ** 15, 2 ** 15)) == 0           # 2^31 voxels
    assert T.tern_packed_bytes((2 ** 16, 1, 2 ** 15, 1, 1)) == 0           # batch counts too
    assert L.tern_pack(fake, Dims(1, 1, 2, 2 ** 15, 2 ** 15), fake, None) == -2
    # output extents are checked as well as input extents (padding grows the output)
    with pytest.raises(T.TernError) as e:
        T.tern_conv_out_dims((1, 1, 1, 1, 2 ** 31 - 2), 1, (1, 1, 1), 1, (0, 0, 1), 1)
    assert e.value.status == -2
    # kernel volume x C_in bounds |accumulator|: it must stay below 2^24
    assert T.tern_filter_bank_bytes(1, 2 ** 14, (16, 8, 8)) == 0           # 2^24
    assert T.tern_filter_bank_bytes(1, 2 ** 14 - 1, (16, 8, 8)) > 0
    assert L.tern_conv3d(fake, Dims(1, 2 ** 14, 16, 8, 8), fake, 1, _geom((16, 8, 8), 1, 0, 1),
                         None, None, fake, None, None) == -2
    # kernel, stride, dilation extents above 1024 are rejected as arguments
    assert L.tern_conv3d(fake, Dims(1, 1, 2000, 4, 4), fake, 1, _geom((1025, 1, 1), 1, 0, 1),
                         None, None, fake, None, None) == -3
    # output channel count
    assert T.tern_filter_bank_bytes(2 ** 19, 1, 1) > 0
    assert T.tern_filter_bank_bytes(2 ** 19 + 1, 1, 1) == 0


def test_unet_entry_points_reject_bad_arguments(T):
    """tern_concat / tern_conv3d_real validate on the host before anything is launched;
    tern_fold_avgpool runs on the host entirely."""
    import numpy as np
    from paper_1801_09449_amd.binding import Dims, Source, _geom
    L = T.lib()
    fake = 0x1000

    def src(c, d=2, h=4, w=4, n=1, up=(1, 1, 1), first=(0, 0, 0), ptr=fake):
        s = Source()
        s.packed = ptr
        s.dims = Dims(n, c, d, h, w)
        for a in range(3):
            s.up[a] = up[a]
            s.first[a] = first[a]
        return s

    out = C.c_void_p(fake)
    one = (Source * 1)(src(8))
    assert L.tern_concat(one, 1, Dims(1, 8, 2, 4, 4), None, None) == -1
    assert L.tern_concat(None, 1, Dims(1, 8, 2, 4, 4), out, None) == -1
    assert L.tern_concat(one, 0, Dims(1, 8, 2, 4, 4), out, None) == -3
    assert L.tern_concat(one, 9, Dims(1, 8, 2, 4, 4), out, None) == -3
    assert L.tern_concat(one, 1, Dims(1, 9, 2, 4, 4), out, None) == -3          # channel sum mismatch
    assert L.tern_concat(one, 1, Dims(2, 8, 2, 4, 4), out, None) == -3          # batch mismatch
    assert L.tern_concat(one, 1, Dims(1, 8, 2, 5, 4), out, None) == -3          # runs past the source
    assert L.tern_concat(one, 1, Dims(1, 8, 0, 4, 4), out, None) == -2
    assert L.tern_concat((Source * 1)(src(8, up=(1, 0, 1))), 1, Dims(1, 8, 2, 4, 4), out, None) == -3
    assert L.tern_concat((Source * 1)(src(8, first=(0, -1, 0))), 1, Dims(1, 8, 2, 4, 4), out, None) == -3
    assert L.tern_concat((Source * 1)(src(8, ptr=None)), 1, Dims(1, 8, 2, 4, 4), out, None) == -1
    assert L.tern_concat((Source * 1)(src(8, ptr=0x1004)), 1, Dims(1, 8, 2, 4, 4), out, None) == -3
    # upsampled source with crop: 2*4 - 1 = 7 rows available from first = 1
    assert L.tern_concat((Source * 1)(src(8, up=(1, 2, 2), first=(0, 1, 1))), 1, Dims(1, 8, 2, 8, 7), out, None) == -3

    g = _geom(3, 1, 0, 1)
    d = Dims(1, 8, 4, 4, 4)
    p = C.c_void_p(fake)
    assert L.tern_conv3d_real(None, d, p, None, 2, g, p, None) == -1
    assert L.tern_conv3d_real(p, d, None, None, 2, g, p, None) == -1
    assert L.tern_conv3d_real(p, d, p, None, 2, g, None, None) == -1
    assert L.tern_conv3d_real(p, d, p, None, 0, g, p, None) == -2
    assert L.tern_conv3d_real(p, Dims(1, 8, 2, 2, 2), p, None, 2, g, p, None) == -2     # kernel does not fit
    assert L.tern_conv3d_real(p, d, C.c_void_p(0x1002), None, 2, g, p, None) == -3      # misaligned weights

    assert L.tern_count_codes(None, d, p, p, None) == -1
    assert L.tern_count_codes(p, d, None, p, None) == -1
    assert L.tern_count_codes(p, Dims(1, 0, 4, 4, 4), p, p, None) == -2
    assert L.tern_count_codes(p, d, C.c_void_p(0x1004), p, None) == -3          # counters need 8-byte alignment

    w = np.arange(2 * 3 * 1 * 2 * 2, dtype=np.int8).reshape(2, 3, 1, 2, 2) % 3 - 1
    f = T.tern_fold_avgpool(w, (1, 2, 3))
    assert f.shape == (2, 3, 1, 4, 6)
    for a in range(4):
        for b in range(6):
            assert (f[:, :, 0, a, b] == w[:, :, 0, a // 2, b // 3]).all()
    with pytest.raises(T.TernError) as e:
        T.tern_fold_avgpool(w, (1, 0, 1))
    assert e.value.status == -3
    with pytest.raises(T.TernError) as e:
        T.tern_fold_avgpool(np.zeros((1, 1, 600, 1, 1), np.int8), (2, 1, 1))    # folded extent above 1024
    assert e.value.status == -2


def test_net_forward_wiring_is_validated_on_the_host(T):
    from paper_1801_09449_amd.binding import Dims, Geom, Module, _geom
    L = T.lib()
    fake = 0x1000
    p = C.c_void_p(fake)

    def mod(c_out, k=3, stride=1, pad=1, skip=-1, up=(1, 1, 1), bank=fake, pool=(1, 1, 1)):
        m = Module(c_out, _geom(k, stride, pad, 1), bank, fake, fake, skip)
        for a in range(3):
            m.up[a] = up[a]
            m.pool[a] = pool[a]
        return m

    d = Dims(1, 4, 4, 8, 8)
    ok = (Module * 3)(mod(8), mod(16, stride=2), mod(8, skip=0, up=(2, 2, 2)))
    need = L.tern_net_workspace_bytes(d, ok, 3)
    # packed input + 3 outputs + one concatenated tensor (8 + 16 channels at the input extent)
    assert need == 256 * 8 + 256 * 8 + 32 * 8 + 256 * 8 + 256 * 8
    assert L.tern_net_workspace_bytes(d, (Module * 1)(mod(8, skip=0)), 1) == 0          # skip from itself
    assert L.tern_net_workspace_bytes(d, (Module * 2)(mod(8), mod(8, skip=1)), 2) == 0   # skip from later
    assert L.tern_net_workspace_bytes(d, (Module * 2)(mod(8), mod(8, up=(0, 1, 1))), 2) == 0
    # the skipped tensor must be at least as large as the (upsampled) incoming one
    assert L.tern_net_workspace_bytes(d, (Module * 3)(mod(8, stride=2), mod(8), mod(8, skip=0, up=(4, 4, 4))), 3) == 0
    # sum pooling in front of a module: a region for the two-digit tensor (64 channels per input
    # word, here 8 channels -> 64, at the pooled extent 4x4x4) on top of input and two outputs
    pooled = (Module * 2)(mod(8), mod(16, pool=(1, 2, 2)))
    assert L.tern_net_workspace_bytes(d, pooled, 2) == 256 * 8 + 256 * 8 + 64 * 16 + 64 * 8
    assert L.tern_net_workspace_bytes(d, (Module * 2)(mod(8), mod(16, pool=(2, 2, 2))), 2) == 0   # window above 4 voxels
    assert L.tern_net_workspace_bytes(d, (Module * 2)(mod(8), mod(16, pool=(1, 5, 1))), 2) == 0
    assert L.tern_net_workspace_bytes(d, (Module * 2)(mod(8), mod(16, pool=(1, -1, 2))), 2) == 0
    hg = _geom(1, 1, 0, 1)
    hd = Dims()
    args = lambda mods, n, ws_bytes, ws=p, head=None, hout=None: L.tern_net_forward(
        p, d, p, p, mods, n, head, None, 2, hg, ws, ws_bytes, hout, C.byref(hd), None, None, None)
    assert args(ok, 3, need - 1) == -4
    assert args(ok, 3, need, ws=C.c_void_p(0x1008)) == -4
    assert args(ok, 3, need, ws=None) == -1
    assert args(ok, 3, need, head=p, hout=None) == -1                                    # head without output
    assert args((Module * 1)(mod(8, bank=None)), 1, need) == -1
    assert args(ok, 0, need) == -3
