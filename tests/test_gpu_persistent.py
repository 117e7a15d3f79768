"""The persistent-workgroup form of the tiled convolution kernel (tuning option, off by default):
the same integers as the oracle, and the plan query says which kernel an input reached."""
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


def check_case(G, c):
    acc, packed = G.run_case(c)
    want = oracle.conv3d(c.act, c.wgt, ConvGeom(c.k, c.stride, c.pad, c.dil))
    np.testing.assert_array_equal(acc, want)
    np.testing.assert_array_equal(packed, oracle.pack(oracle.threshold(want, c.lo, c.hi)))

STREAM = 8   # TERN_OPT_STREAM


@pytest.fixture
def persistent():
    import paper_1801_09449_amd as T
    T.tern_set_option(STREAM, 1)
    yield T
    T.tern_set_option(STREAM, 0)


def test_persistent_kernel_config1_every_output(G, persistent):
    """config[1] (2048 tiles, two per workgroup): int32 and fused outputs, element by element."""
    T = persistent
    check_case(G, synth.config1())
    plan = T.tern_last_launch()
    assert plan["kernel"] == T.KERNEL_PERSISTENT
    assert plan["threads"] == 256 and plan["grid_y"] == 1 and plan["grid_x"] <= 1024


@pytest.mark.parametrize("name,n,c_in,vol", [("ragged", 1, 64, (60, 76, 100)), ("batch_one_word", 3, 32, (48, 48, 48))])
def test_persistent_kernel_ragged_tiles_and_runs_across_batch_items(G, persistent, name, n, c_in, vol):
    """Extents that leave partial tiles on every axis and an uneven run of tiles for the last
    workgroup; a batch whose workgroups walk from one item into the next, one word per voxel."""
    T = persistent
    check_case(G, synth.conv_case("pw_" + name, n, c_in, 64, vol, seed=611, p0_a=0.4))
    assert T.tern_last_launch()["kernel"] == T.KERNEL_PERSISTENT


def test_persistent_kernel_on_a_stack_of_planes(G, persistent):
    """Kernel depth 1 on a batch of single-plane inputs: the batch collapses into planes, a wave
    covers 4 x 8 voxels in two planes, and four waves of a workgroup take four channel slices."""
    T = persistent
    check_case(G, synth.conv_case("pw_planes", 32, 128, 128, (1, 116, 84), k=(1, 3, 3), pad=0, seed=614, p0_a=0.4))
    plan = T.tern_last_launch()
    assert plan["kernel"] == T.KERNEL_PERSISTENT, sorted(plan.items())


def test_option_leaves_ineligible_launches_to_the_other_kernels(G, persistent):
    """Too few tiles, channel counts that need several workgroups per tile, single taps: the
    option changes nothing there."""
    T = persistent
    check_case(G, synth.conv_case("pw_small", 1, 64, 64, (16, 16, 16), seed=612))
    assert T.tern_last_launch()["kernel"] == T.KERNEL_TILED
    check_case(G, synth.conv_case("pw_k1", 1, 64, 64, (16, 16, 16), k=1, pad=0, seed=613))
    assert T.tern_last_launch()["kernel"] == T.KERNEL_POINTWISE


def test_default_launch_of_config1_is_one_workgroup_per_tile(G):
    import paper_1801_09449_amd as T
    c = synth.config1()
    a = T.tern_pack(G.dev(c.act))
    T.tern_conv3d(a, 64, T.tern_pack_filters(G.dev(c.wgt)), 64, thr_lo=G.dev(c.lo), thr_hi=G.dev(c.hi))
    plan = T.tern_last_launch()
    assert plan == {"kernel": T.KERNEL_TILED, "voxels_per_lane": 1, "channels_per_pass": 32, "tap_split": 1,
                    "threads": 256, "grid_x": 2048, "grid_y": 1, "lds_bytes": 6400}


def test_tuning_options_belong_to_the_calling_thread(G):
    """An override set by one host thread changes neither the plan nor the options of another."""
    import threading
    import torch
    import paper_1801_09449_amd as T
    c = synth.conv_case("thr", 1, 64, 64, (32, 64, 64), seed=615)
    a = T.tern_pack(G.dev(c.act))
    bank = T.tern_pack_filters(G.dev(c.wgt))
    lo, hi = G.dev(c.lo), G.dev(c.hi)
    run = lambda: T.tern_conv3d(a, 64, bank, 64, thr_lo=lo, thr_hi=hi)
    plans = {}

    def worker():
        plans["before"] = T.tern_last_launch()["kernel"]     # nothing launched by this thread yet
        plans["other"] = (run(), T.tern_last_launch())[1]

    T.tern_set_option(3, 16)      # TERN_OPT_CO_BLOCK
    try:
        mine_forced = (run(), T.tern_last_launch())[1]
        th = threading.Thread(target=worker)
        th.start(); th.join()
    finally:
        T.tern_set_option(3, 0)
    mine_default = (run(), T.tern_last_launch())[1]
    torch.cuda.synchronize()
    assert plans["before"] == -1
    assert mine_forced["channels_per_pass"] == 16
    assert plans["other"]["channels_per_pass"] == 32 and plans["other"] == mine_default
