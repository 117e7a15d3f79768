#!/usr/bin/env python3
"""Benchmark of the ternary 3D convolution on one MI355X.

One step = one call of the fused ternary convolution (halo staging, masked-Hamming contraction,
threshold + re-pack epilogue) on BASELINE config[1]: batch 1, C_in = C_out = 64, 64^3 volume, 3^3
kernel, stride 1, pad 1, seeded synthetic ternary data already resident in HBM and already packed
(as it is between layers of a network).  Prints ONE JSON line.

Besides the headline the line carries: the roofline of the timed kernel (issued vector
instructions against the ALU ceiling derived from unit counts and clock, with the rate of the same
instruction sequence measured in this run beside it), a
check of the timed output against the CPU oracle, per-launch statistics, one compact row for each
of the other BASELINE configurations, and the oracle timed on the host cores.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Vector-ALU ceiling of the kernel's instruction mix, from unit counts and clock: 256 compute
# units x 4 SIMDs at 2.4 GHz.  A SIMD retires a wave-wide integer instruction on vector registers
# in two cycles (32 lanes per clock: the rate behind the published 157.3 TFLOP/s of fp32 vector
# arithmetic), v_bcnt_u32_b32 in four (half rate, like fp64), and an instruction with a scalar-
# register operand occupies the operand bus for four but the ALU for two.  A ternary word pair
# (and, popcount-accumulate, three-input bit op, popcount-accumulate) is 2 + 4 + 2 + 4 = 12 ALU
# cycles, 3.0 per instruction; a binary one (bit op, popcount-accumulate) 6.  tern_probe_valu
# measures every one of these rates (variants 2-16) and the sequences themselves (0, 10).
SIMDS, CLOCK_HZ = 256 * 4, 2.4e9
PEAK_LANE_OPS_TERNARY = SIMDS * CLOCK_HZ / 3.0 * 64      # 52.43e12 issued lane-ops/s = 419 TMAC/s
PEAK_LANE_OPS_BINARY = SIMDS * CLOCK_HZ / 3.0 * 64       # 2 instructions in 6 cycles: the same 3.0
NOMINAL_LANE_OPS = 256 * 64 * 2.4e9       # 39.32e12: one wave instruction per SIMD every four cycles
# The kernels issue four vector instructions per 32-bit word pair (32 MACs): and, popcount-
# accumulate, three-input bit operation, popcount-accumulate.  Counted from the kernel's code: 94.5 %
# of the instructions of a config[1] wave are these.
ISSUED_OPS_PER_MAC = 4.0 / 32.0
# The method as the paper writes it needs five operations per word pair (and, xor, and, two
# popcount-accumulates); kept as a secondary figure beside the issued-instruction count.
ALGORITHMIC_OPS_PER_MAC = 5.0 / 32.0
# HBM bytes per launch of the config[1] kernel: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by
# a 256 MiB copy under the same counters (profiles/conv3d_fused_config1.md).  A profiler figure,
# not measured by this script.
TRAFFIC_BYTES_CFG1 = 10.09e6
ALGORITHMIC_BYTES_CFG1 = 8.42e6
SETTLE_MS = 40.0                          # GPU work in front of every timed region (clocks settle)


def settle(fn, min_ms=SETTLE_MS, max_ms=400.0):
    """Run fn back to back until its time per launch has stopped falling: at least min_ms of GPU
    time, whatever --warmup says, then on until four bursts in a row agree within 1 % (or max_ms).
    After an idle period (input generation on the host) the shader clock comes back over tens of
    milliseconds of load: config[1] launches take 101 us at first, 95 us after 45 ms on some
    boxes, 88-91 us from then on; a pause of a millisecond does not undo that, one of 20 ms does.
    A 2 ms timed region right after an idle period measures that ramp, not the kernel.  Bursts of
    50 launches with a synchronisation between them: the pauses are tens of microseconds, and the
    launch queue stays short."""
    import torch
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total, per = 0.0, []
    while total < max_ms:
        ev0.record()
        for _ in range(50):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        t = ev0.elapsed_time(ev1)
        total += t
        per.append(t)
        if total >= min_ms and len(per) >= 4 and max(per[-4:]) <= 1.01 * min(per[-4:]):
            break
    return total


def timed(fn, steps, warmup, stream_sync=None, settle_first=True):
    """Average milliseconds per call by events on the current stream, plus wall time."""
    import torch
    if settle_first:
        timed.last_settle_ms = settle(fn)
        # One rehearsal of the timed region itself (synchronise, event, the same number of
        # launches, event, synchronise), not counted: the first such region of a process has
        # measured 5-40 us per launch longer than every later one (the host falls behind the GPU
        # once while the queue is still empty), which a 20-launch region cannot absorb.
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record()
        for _ in range(steps):
            fn()
        r1.record()
        torch.cuda.synchronize()
        r0.elapsed_time(r1)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        fn()
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return ev0.elapsed_time(ev1) / steps, wall


def graph_ms(fn, calls=20, reps=30):
    """Milliseconds of GPU time per call with `calls` calls recorded into one HIP graph and the
    graph replayed: what a launch costs without the binding's host work per call."""
    import torch
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(calls):
            fn()
    settle(g.replay)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        g.replay()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / reps / calls


def per_launch(fn, count):
    """Milliseconds of `count` single launches, each bracketed by its own pair of events."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def cpu_baseline(case, target_seconds=12.0):
    """The oracle, as it stands, timed on the host cores on a z-slab of the same workload sized
    to about target_seconds.  Returns the JSON object and (accumulators, input planes used)."""
    import numpy as np
    import oracle
    from oracle import ConvGeom
    g = ConvGeom(case.k, case.stride, case.pad, case.dil)
    d = case.act.shape[2]
    probe = min(d, 4)
    sub = np.ascontiguousarray(case.act[:, :, :probe])
    t0 = time.perf_counter()
    oracle.conv3d(sub, case.wgt, g)
    dt = time.perf_counter() - t0
    per_plane = dt / probe
    planes = int(max(probe, min(d, target_seconds / max(per_plane, 1e-9))))
    sub = np.ascontiguousarray(case.act[:, :, :planes])
    t0 = time.perf_counter()
    acc = oracle.conv3d(sub, case.wgt, g)
    dt = time.perf_counter() - t0
    macs = acc.size * case.act.shape[1] * case.k[0] * case.k[1] * case.k[2]
    return {
        "value": macs / dt / 1e12, "unit": "TMAC/s", "cores": oracle.max_threads(), "kind": "oracle",
        "sample": f"z-slab of {planes} of {d} input planes of config[1] (same channels and kernel), "
                  f"1 repetition, {dt:.2f} s",
    }, acc, planes


def check_against_oracle(case, out_packed, acc_slab, planes):
    """The timed call's packed output against the oracle.  With the accumulators of a z-slab of the
    input (from cpu_baseline): every output plane whose taps lie inside the slab, all channels and
    voxels.  Without: 4096 sampled outputs through the oracle's point evaluation."""
    import numpy as np
    import oracle
    from oracle import ConvGeom
    got = out_packed.cpu().numpy().view(np.uint32)            # [1][D][H][W][2][Wd]
    d = case.act.shape[2]
    if acc_slab is not None:
        # an output plane z of the slab run equals the full run's when z + pad < planes (or the
        # slab is the whole volume)
        good = d if planes >= d else max(0, planes - case.pad[0] * case.dil[0])
        want = oracle.pack(oracle.threshold(np.ascontiguousarray(acc_slab[:, :, :good]), case.lo, case.hi))
        ok = bool(np.array_equal(got[:, :good], want))
        return ok, f"{good} of {d} output planes, every voxel and channel, against oracle conv3d + threshold + pack"
    rng = np.random.default_rng(0)
    od, oh, ow = case.out_spatial
    c_out = case.wgt.shape[0]
    pts = np.stack([np.zeros(4096, np.int64), rng.integers(0, c_out, 4096), rng.integers(0, od, 4096),
                    rng.integers(0, oh, 4096), rng.integers(0, ow, 4096)], axis=1).astype(np.int32)
    acc = oracle.conv3d_points(case.act, case.wgt, ConvGeom(case.k, case.stride, case.pad, case.dil), pts)
    code = np.where(acc > case.hi[pts[:, 1]], 1, np.where(acc < case.lo[pts[:, 1]], -1, 0))
    w = got[0, pts[:, 2], pts[:, 3], pts[:, 4]]                # [P][2][Wd]
    q, b = pts[:, 1] // 32, pts[:, 1] % 32
    m = (w[np.arange(4096), 0, q] >> b.astype(np.uint32)) & 1
    sg = (w[np.arange(4096), 1, q] >> b.astype(np.uint32)) & 1
    got_code = np.where(m == 0, 0, np.where(sg == 1, -1, 1))
    return bool(np.array_equal(got_code, code)), "4096 sampled outputs against oracle conv3d_points + Eq. 6"


def conv_times(T, dev, c, steps=30, warmup=5):
    """(fused ms, int32-output ms) of one single-layer case."""
    import torch
    c_in, c_out = c.act.shape[1], c.wgt.shape[0]
    a = T.tern_pack(dev(c.act))
    bank = T.tern_pack_filters(dev(c.wgt))
    lo, hi = dev(c.lo), dev(c.hi)
    g = dict(k=c.k, stride=c.stride, pad=c.pad, dil=c.dil)
    outp = T.tern_conv3d(a, c_in, bank, c_out, thr_lo=lo, thr_hi=hi, **g)
    outa = T.tern_conv3d(a, c_in, bank, c_out, **g)
    ms_f, _ = timed(lambda: T.tern_conv3d(a, c_in, bank, c_out, thr_lo=lo, thr_hi=hi, out=outp, **g), steps, warmup, None)
    ms_a, _ = timed(lambda: T.tern_conv3d(a, c_in, bank, c_out, out=outa, **g), steps, warmup, None)
    del a, bank, outp, outa
    torch.cuda.empty_cache()
    return ms_f, ms_a


def extras(T, synth, dev, case, act_i8, act, bank, lo, hi, out_acc, out_packed, geom):
    """Timings of the other entry points and of the other BASELINE configurations."""
    import numpy as np
    import torch
    c_in, c_out = case.act.shape[1], case.wgt.shape[0]
    ex = {}
    ms_acc, _ = timed(lambda: T.tern_conv3d(act, c_in, bank, c_out, out=out_acc, **geom), 50, 5, None)
    ex["cfg1_conv3d_int32_out_ms"] = ms_acc
    # the persistent-workgroup form of the tiled kernel (tuning option 8, off by default) beside
    # the default launch, on the shapes it applies to
    c4d1 = [c for c in synth.config4_cases() if c.name == "cfg4_k3_d1_pw0.5"][0]
    pw = {}
    for name, c in (("cfg1", case), ("cfg4_k3_d1", c4d1),
                    ("batch3_48cubed_32_to_64", synth.conv_case("pw_b", 3, 32, 64, 48, seed=8, p0_a=0.4))):
        row = {}
        for label, opt in (("default", 0), ("persistent", 1)):
            T.tern_set_option(8, opt)
            try:
                f, a = conv_times(T, dev, c, steps=50, warmup=5)
                row[label + "_kernel"] = T.tern_last_launch()["kernel"]
            finally:
                T.tern_set_option(8, 0)
            row[label + "_fused_ms"] = f
            row[label + "_int32_ms"] = a
        pw[name] = row
    ex["persistent_workgroups"] = pw
    ms_pack, _ = timed(lambda: T.tern_pack(act_i8, out=act), 50, 5, None)
    ex["cfg1_pack_i8_ms"] = ms_pack
    ex["cfg1_pack_i8_GBps"] = (act_i8.numel() + act.numel() * 4) / (ms_pack * 1e-3) / 1e9
    ms_thr, _ = timed(lambda: T.tern_threshold_pack(out_acc, lo, hi, out=out_packed), 50, 5, None)
    ex["cfg1_threshold_pack_i32_ms"] = ms_thr
    ex["cfg1_threshold_pack_i32_GBps"] = (out_acc.numel() * 4 + out_packed.numel() * 4) / (ms_thr * 1e-3) / 1e9

    def row(c):
        f, a = conv_times(T, dev, c)
        return {"gmac": c.macs / 1e9, "fused_ms": f, "int32_ms": a, "fused_TMACs": c.macs / (f * 1e-3) / 1e12,
                "int32_TMACs": c.macs / (a * 1e-3) / 1e12}
    ex["cfg0"] = row(synth.config0())
    ex["cfg3"] = row(synth.config3())
    for c in synth.config4_cases():
        if c.meta["p0_w"] == 0.5:
            ex[c.name] = row(c)

    f = synth.config2()
    layers = [T.FcnLayer(L["w"].shape[1], L["w"].shape[0], T.tern_pack_filters(dev(L["w"])),
                         dev(L["lo"]), dev(L["hi"]), L["k"], L["stride"], L["pad"], L["dil"])
              for L in f.layers]
    x, ilo, ihi = dev(f.x), dev(f.in_lo), dev(f.in_hi)
    ws = torch.empty((T.tern_fcn_workspace_bytes(x.shape, layers),), dtype=torch.uint8, device="cuda")
    out = T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws)
    ms_fcn, _ = timed(lambda: T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws, out=out), 30, 5, None)
    ex["cfg2_fcn"] = {"gmac": f.macs / 1e9, "ms": ms_fcn, "TMACs": f.macs / (ms_fcn * 1e-3) / 1e12}
    # the same chain recorded once into a HIP graph and replayed (no per-launch host work)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws, out=out)
    ms_g, _ = timed(graph.replay, 30, 5, None)
    ex["cfg2_fcn"]["graph_replay_ms"] = ms_g
    # per layer
    cur = tuple(x.shape)
    a_in = T.tern_threshold_pack(x, ilo, ihi)
    per = []
    for L in layers:
        o = T.tern_conv3d(a_in, L.c_in, L.w_bank, L.c_out, L.k, L.stride, L.pad, L.dil, thr_lo=L.thr_lo, thr_hi=L.thr_hi)
        ms_l, _ = timed(lambda: T.tern_conv3d(a_in, L.c_in, L.w_bank, L.c_out, L.k, L.stride, L.pad, L.dil,
                                              thr_lo=L.thr_lo, thr_hi=L.thr_hi, out=o), 30, 5, None)
        per.append(round(ms_l, 5))
        a_in = o
    ex["cfg2_fcn"]["layer_ms"] = per
    ms_in, _ = timed(lambda: T.tern_threshold_pack(x, ilo, ihi), 30, 5, None)
    ex["cfg2_fcn"]["input_threshold_pack_ms"] = ms_in
    # the same encoder as a chain of tern_net_forward modules
    mods = [T.NetModule(L["w"].shape[0], T.tern_pack_filters(dev(L["w"])), dev(L["lo"]), dev(L["hi"]), k=L["k"],
                        stride=L["stride"], pad=L["pad"], dil=L["dil"]) for L in f.layers]
    ws_n = torch.empty((T.tern_net_workspace_bytes(x.shape, mods),), dtype=torch.uint8, device="cuda")
    ms_n, _ = timed(lambda: T.tern_net_forward(x, ilo, ihi, mods, workspace=ws_n), 30, 5, None)
    ex["cfg2_net_forward_ms"] = ms_n

    # The paper's baseline U-Net (Table 1) on synthetic weights, whole forward pass, for one
    # stack of slices and for a batch of 16 stacks.  MACs in the paper's convention (a pooled
    # module counted at the pooled resolution) and as executed (pooling folded into the filters
    # repeats every tap over the pooling window: 4 x; pooling into two digits: 2 x).
    from paper_1801_09449_amd import unet
    for n in (1, 16):
        u = synth.unet_table1(seed=0, n=n)
        plan = unet.UNetPlan(u.layers, u.head_w, u.head_b, u.in_lo, u.in_hi)
        ux = dev(u.x)
        pred, kept = unet.unet_forward(plan, ux, keep_layers=True)
        nominal = executed = 0
        chosen = plan.modules(ux.shape)
        for L, (t, c), m in zip(u.layers, kept, chosen):
            vox = t.shape[0] * t.shape[1] * t.shape[2] * t.shape[3]
            taps = int(np.prod(L["k"]))
            nominal += vox * c * L["w"].shape[1] * taps
            if max(m.pool) > 1:      # two digits: the channel words double
                executed += vox * c * 64 * ((L["w"].shape[1] + 31) // 32) * taps
            else:
                executed += vox * c * L["w"].shape[1] * taps * (int(np.prod(L["pool"])) if L["pool"] else 1)
        del kept
        ms_u, _ = timed(lambda: unet.unet_forward(plan, ux, out=pred), 20, 3, None)
        ugraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(ugraph):
            unet.unet_forward(plan, ux, out=pred)
        ms_ug, _ = timed(ugraph.replay, 20, 3, None)
        ex["unet_table1_n%d" % n] = {"ms": ms_u, "graph_replay_ms": ms_ug,
                                     "gmac_table1_convention": nominal / 1e9,
                                     "gmac_executed": executed / 1e9,
                                     "TMACs_executed": executed / (ms_u * 1e-3) / 1e12,
                                     "prediction_shape": list(pred.shape)}
    # the matrix-instruction experiment (include/tern_matrix.h), beside the contract's path
    c4 = {c.name: c for c in synth.config4_cases()}
    for name, c in (("cfg1", case), ("cfg3", synth.config3()), ("cfg4_k3_d1_pw0.5", c4["cfg4_k3_d1_pw0.5"]),
                    ("cfg4_k3_d3_pw0.5", c4["cfg4_k3_d3_pw0.5"])):
        ci, co = c.act.shape[1], c.wgt.shape[0]
        g = dict(k=c.k, stride=c.stride, pad=c.pad, dil=c.dil)
        a_p = T.tern_pack(dev(c.act)); l_, h_ = dev(c.lo), dev(c.hi)
        row = {}
        for kind in ("i8", "f4"):
            mb = T.tern_expand_filters(dev(c.wgt), kind)
            o = T.tern_conv3d(a_p, ci, mb, co, thr_lo=l_, thr_hi=h_, mfma=kind, **g)
            ms_k, _ = timed(lambda: T.tern_conv3d(a_p, ci, mb, co, thr_lo=l_, thr_hi=h_, mfma=kind, out=o, **g), 30, 5, None)
            row[kind] = {"ms": ms_k, "TMACs": c.macs / (ms_k * 1e-3) / 1e12}
        ex["mfma_" + name] = row
    return ex


def config_rows(T, synth, dev, peak_issue):
    """One compact row per other BASELINE configuration (fused call, HBM-resident packed input)."""
    import numpy as np
    import torch
    rows = {}

    def row(c, steps=30):
        f, a = conv_times(T, dev, c, steps=steps, warmup=3)
        r = {"gmac": round(c.macs / 1e9, 3), "fused_ms": round(f, 5), "int32_out_ms": round(a, 5),
             "TMACs": round(c.macs / (f * 1e-3) / 1e12, 2)}
        if peak_issue:
            r["issued_frac_of_alu_peak"] = round(ISSUED_OPS_PER_MAC * c.macs / (f * 1e-3) / peak_issue, 3)
        return r

    rows["config0"] = row(synth.config0(), steps=100)
    # config[0] is shorter than the binding's host work per call: GPU time per launch from a
    # replayed graph of 20 calls
    c0 = synth.config0()
    a0, b0 = T.tern_pack(dev(c0.act)), T.tern_pack_filters(dev(c0.wgt))
    l0, h0 = dev(c0.lo), dev(c0.hi)
    g0 = dict(k=c0.k, stride=c0.stride, pad=c0.pad, dil=c0.dil)
    o0 = T.tern_conv3d(a0, 32, b0, 32, thr_lo=l0, thr_hi=h0, **g0)
    rows["config0"]["fused_graph_replay_ms"] = round(
        graph_ms(lambda: T.tern_conv3d(a0, 32, b0, 32, thr_lo=l0, thr_hi=h0, out=o0, **g0)), 5)
    del a0, b0, o0
    f = synth.config2()
    layers = [T.FcnLayer(L["w"].shape[1], L["w"].shape[0], T.tern_pack_filters(dev(L["w"])),
                         dev(L["lo"]), dev(L["hi"]), L["k"], L["stride"], L["pad"], L["dil"])
              for L in f.layers]
    x, ilo, ihi = dev(f.x), dev(f.in_lo), dev(f.in_hi)
    ws = torch.empty((T.tern_fcn_workspace_bytes(x.shape, layers),), dtype=torch.uint8, device="cuda")
    out = T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws)
    ms_fcn, _ = timed(lambda: T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws, out=out), 30, 3)
    ms_fcn_g = graph_ms(lambda: T.tern_fcn_forward(x, ilo, ihi, layers, workspace=ws, out=out), calls=5)
    rows["config2"] = {"gmac": round(f.macs / 1e9, 3), "fused_ms": round(ms_fcn, 5),
                       "fused_graph_replay_ms": round(ms_fcn_g, 5),
                       "TMACs": round(f.macs / (ms_fcn * 1e-3) / 1e12, 2),
                       "what": "tern_fcn_forward: float input, Eq. 6, six fused layers"}
    del x, ws, out, layers
    rows["config3"] = row(synth.config3())
    for c in synth.config4_cases():
        if c.meta["p0_w"] == 0.5:
            rows["config4_" + c.name[5:].replace("_pw0.5", "")] = row(c)
    torch.cuda.empty_cache()
    return rows


def binary_row(T, synth, dev, probe_rate):
    """The binary special case (Eq. 8) at config[1]'s shape on inputs without zeros: two issued
    vector instructions per word pair against the rate of that pair in a register-only loop."""
    import torch
    c = synth.conv_case("cfg1_binary", 1, 64, 64, 64, p0_w=0.0, p0_a=0.0, seed=0, thr_range=(-24, 24))
    a = T.tern_pack(dev(c.act))
    bank = T.tern_pack_filters_binary(dev(c.wgt))
    lo, hi = dev(c.lo), dev(c.hi)
    out = T.tern_conv3d_binary(a, 64, bank, 64, thr_lo=lo, thr_hi=hi)
    ms, _ = timed(lambda: T.tern_conv3d_binary(a, 64, bank, 64, thr_lo=lo, thr_hi=hi, out=out), 100, 5)
    peak = probe_rate(10)
    issued = (2.0 / 32.0) * c.macs / (ms * 1e-3)
    torch.cuda.synchronize()
    # the same kernel on the shapes of config[3] and config[4] (3^3, dilation 1): longer launches
    larger = {}
    for name, n, ch, vol in (("config3_shape", 2, 256, 32), ("config4_k3_d1_shape", 1, 64, 96)):
        cl = synth.conv_case(name, n, ch, ch, vol, p0_w=0.0, p0_a=0.0, seed=0, thr_range=(-24, 24))
        al, bl = T.tern_pack(dev(cl.act)), T.tern_pack_filters_binary(dev(cl.wgt))
        ll, hl = dev(cl.lo), dev(cl.hi)
        ol = T.tern_conv3d_binary(al, ch, bl, ch, thr_lo=ll, thr_hi=hl)
        ms_l, _ = timed(lambda: T.tern_conv3d_binary(al, ch, bl, ch, thr_lo=ll, thr_hi=hl, out=ol), 30, 3)
        larger[name] = {"gmac": round(cl.macs / 1e9, 3), "fused_ms": round(ms_l, 5),
                        "TMACs": round(cl.macs / (ms_l * 1e-3) / 1e12, 2),
                        "issued_frac_of_alu_peak": round((2.0 / 32.0) * cl.macs / (ms_l * 1e-3) / PEAK_LANE_OPS_BINARY, 3)}
        del al, bl, ol
    torch.cuda.empty_cache()
    return {"workload": "tern_conv3d_binary, config[1]'s shape, +-1 weights and activations, fused cut points",
            "gmac": round(c.macs / 1e9, 3), "fused_ms": round(ms, 5), "TMACs": round(c.macs / (ms * 1e-3) / 1e12, 2),
            "roofline": {"bound": "alu", "achieved": issued / 1e12, "peak": PEAK_LANE_OPS_BINARY / 1e12,
                         "unit": "T lane-op/s", "frac": issued / PEAK_LANE_OPS_BINARY,
                         "basis": "2 issued vector lane-ops per 32 MACs (three-input bit op 2 cycles, popcount-"
                                  "accumulate 4) against 1024 SIMDs x 2.4 GHz x 64 lanes / 3.0 = 839 TMAC/s",
                         "measured_sequence_peak": peak / 1e12, "frac_of_measured_sequence_peak": issued / peak},
            "larger_launches": larger}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the rows of the other configurations")
    ap.add_argument("--extras", action="store_true", help="also time the other entry points")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference for HBM counters)")
    ap.add_argument("--lane-depth", type=int, default=0, help="tuning override: 0 auto, 2 or 4")
    ap.add_argument("--waves-z", type=int, default=0, help="tuning override: 0 auto, 1, 2, 4, 8")
    ap.add_argument("--co-block", type=int, default=0, help="tuning override: 0 auto, 16, 32")
    ap.add_argument("--tap-split", type=int, default=0, help="tuning override: 0 auto, 1, 2, 4, 8")
    ap.add_argument("--co-per-wave", type=int, default=0, help="tuning override: 0 auto, multiple of 16")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); sharding over several "
              "GPUs is not built.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1801_09449_amd as T
    import synth

    T.lib()
    T.tern_set_option(1, args.lane_depth)
    T.tern_set_option(2, args.waves_z)
    T.tern_set_option(3, args.co_block)
    T.tern_set_option(4, args.co_per_wave)
    T.tern_set_option(5, args.tap_split)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    case = synth.config1()
    c_in, c_out = case.act.shape[1], case.wgt.shape[0]
    act_i8 = dev(case.act)
    act = T.tern_pack(act_i8)
    bank = T.tern_pack_filters(dev(case.wgt))
    lo, hi = dev(case.lo), dev(case.hi)
    out_packed = torch.empty_like(act)
    out_acc = torch.empty((1, c_out) + case.out_spatial, dtype=torch.int32, device="cuda")
    geom = dict(k=case.k, stride=case.stride, pad=case.pad, dil=case.dil)

    def step():
        T.tern_conv3d(act, c_in, bank, c_out, thr_lo=lo, thr_hi=hi, out=out_packed, **geom)

    ms, wall_ms = timed(step, args.steps, args.warmup)
    settle_ms = timed.last_settle_ms
    singles = per_launch(step, max(10, min(args.steps, 200)))
    macs = case.macs
    tmacs = macs / (ms * 1e-3) / 1e12
    issued = ISSUED_OPS_PER_MAC * macs / (ms * 1e-3)
    algorithmic = ALGORITHMIC_OPS_PER_MAC * macs / (ms * 1e-3)

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Ceiling: the kernels' own instruction sequence in a register-only loop (no memory, four
    # waves per SIMD), measured here and now; beside it the same four instructions with no scalar
    # instruction between them, and a stream of one plain opcode (the nominal rate).
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    p_blocks, p_threads, p_iters = 8192, 256, 1000

    def probe_rate(variant):
        ms_p, _ = timed(lambda: T.tern_probe_valu(p_blocks, p_threads, p_iters, sink, variant), 3, 1)
        return p_blocks * p_threads * p_iters * 65.0 / (ms_p * 1e-3)

    peak = probe_rate(0)
    result = {
        "metric": "ternary MAC/s (TMAC/s) + ms per volume; % of int/popcount peak",
        "value": tmacs, "unit": "TMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
        "config": {"workload": "config[1]: fused ternary conv3d, N=1, C_in=C_out=64, 64^3, k=3^3, "
                               "s=1, p=1, packed in -> packed out", "gmac": macs / 1e9,
                   "wall_ms_per_step": wall_ms, "settle_ms_before_timing": round(settle_ms, 1),
                   "settle_rule": "at least %g ms, then until four bursts of 50 launches agree within 1 %% (at most 400 ms)" % SETTLE_MS},
        "launch_ms": {"mean": ms, "median": statistics.median(singles), "min": min(singles),
                      "single_launches": len(singles)},
        "roofline": {
            "bound": "alu", "achieved": issued / 1e12, "peak": PEAK_LANE_OPS_TERNARY / 1e12, "unit": "T lane-op/s",
            "frac": issued / PEAK_LANE_OPS_TERNARY,
            "basis": "achieved = 4 issued 32-bit vector lane-ops per 32 MACs (and, popcount-accumulate, "
                     "three-input bit op, popcount-accumulate: the kernel's instructions per word pair) x "
                     "MAC/s; peak = 1024 SIMDs x 2.4 GHz x 64 lanes / 3.0 cycles per instruction (12 ALU cycles "
                     "per word pair: vector-only integer ops 2, v_bcnt_u32_b32 4), i.e. 419 TMAC/s",
            "measured_sequence_peak": peak / 1e12,
            "frac_of_measured_sequence_peak": issued / peak,
            "measured_basis": "the kernels' own word-pair sequence in a register-only loop, four waves per SIMD, "
                              "timed in this run (tern_probe_valu variant 0)",
            "probe_cycles_per_instruction": {name: SIMDS * CLOCK_HZ * 64 / probe_rate(v) for name, v in (
                ("kernel_sequence", 0), ("same_instructions_no_scalar_spacer", 1), ("v_and_b32_scalar_operand", 2),
                ("v_bcnt_u32_b32", 4), ("v_bitop3_b32_scalar_operand", 6), ("v_xor_b32_vector_only", 14),
                ("v_bitop3_b32_vector_only", 15), ("scalar_operand_and_beside_vector_only_add", 16))},
            "one_instruction_per_four_cycles": {"rate": NOMINAL_LANE_OPS / 1e12,
                                                "issued_frac": issued / NOMINAL_LANE_OPS,
                                                "algorithmic_5op_frac": algorithmic / NOMINAL_LANE_OPS,
                                                "note": "256 CU x 64 lanes x 2.4 GHz is not a ceiling for integer "
                                                        "ops on vector registers (they retire in two cycles); the "
                                                        "paper's five operations per word pair against it exceed 1"},
            "traffic": TRAFFIC_BYTES_CFG1,
            "traffic_basis": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel, profiles/conv3d_fused_config1.md "
                             "(a profiler run of the same command, not this run)",
            "algorithmic_bytes": ALGORITHMIC_BYTES_CFG1,
            "hbm_GBps": TRAFFIC_BYTES_CFG1 / (ms * 1e-3) / 1e9,
        },
    }

    if not args.no_configs:
        result["configs"] = config_rows(T, synth, dev, PEAK_LANE_OPS_TERNARY)
        result["binary_eq8"] = binary_row(T, synth, dev, probe_rate)

    if args.extras:
        result["extras"] = extras(T, synth, dev, case, act_i8, act, bank, lo, hi, out_acc, out_packed, geom)

    # the timed call's output against the oracle
    step()
    torch.cuda.synchronize()
    acc_slab, planes = None, 0
    if not args.no_cpu_baseline:
        result["cpu_baseline"], acc_slab, planes = cpu_baseline(case)
        import oracle
        c0 = synth.config0()
        from oracle import ConvGeom
        all_threads = oracle.max_threads()
        oracle.set_threads(1)
        t0 = time.perf_counter()
        oracle.conv3d(c0.act, c0.wgt, ConvGeom(c0.k, c0.stride, c0.pad, c0.dil))
        dt0 = time.perf_counter() - t0
        oracle.set_threads(all_threads)
        result["cpu_baseline"]["config0_single_thread"] = {"seconds": dt0, "TMACs": c0.macs / dt0 / 1e12}
    ok, how = check_against_oracle(case, out_packed, acc_slab, planes)
    result["parity_checked"] = ok
    result["parity_check"] = how
    print(json.dumps(result))
    if not ok:
        print("bench.py: the timed output differs from the oracle", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
