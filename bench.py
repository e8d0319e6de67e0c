#!/usr/bin/env python3
"""Benchmark of the table-lookup hot path on one MI355X.

A "step" is one pass of the whole path over one batch that is already resident in HBM:
quantise the fp32 input -> approximate layer(s) -> dequantise (+ the fp32 glue of the network
configurations).  Default workload: the 3x3 convolution layer the metric is quoted on
(batch 32, 64 -> 64 channels, 32x32, 8-bit table).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1|2|3|4|5] [--bits B] [--no-cpu-baseline]
                  [--copy-calibration]

Configurations 6 - 11 are workloads beyond the five baseline ones (separable block, GRU, 12-bit operands, the
straight-through backward pass of a linear and of a convolution layer); they print the same line with their own metric.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

LDS_LANES_PER_CLK_PER_CU = 32      # 32 banks x 4 B: one 16-bit gather lane per bank per clock (the model peak named for this path)
MODEL_CLOCK_GHZ = 2.4
GATHER_LANES_PER_CLK_PER_CU = 4    # vector memory path: one 64-lane gather instruction per 16 clocks
MITCHELL_OPS_PER_MAC = 15          # vector instructions per multiply-accumulate counted in the compiled function-form kernel (484 per 32)
MODEL_CUS = 256
HBM_PEAK_BYTES_PER_S = 8.0e12      # published HBM3E rate of MI355X

# HBM traffic of the headline configuration's kernels: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries (KiB per
# dispatch) and the same counters for a plain copy of known size, which they are scaled by (commands inside the file)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_config2.txt")


def read_traffic():
    """{kernel: HBM bytes per dispatch} from the committed counter summary, or {} when there is none."""
    vals = {}
    try:
        for line in open(TRAFFIC_FILE):
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                vals[k.strip()] = float(v)
    except OSError:
        return {}
    try:
        f_scale = vals["copy_kib"] / vals["copy_fetch_kib"]
        w_scale = vals["copy_kib"] / vals["copy_write_kib"]
    except (KeyError, ZeroDivisionError):
        return {}
    out = {}
    for k in vals:
        if k.endswith("_fetch_kib") and not k.startswith("copy_"):
            name = k[:-len("_fetch_kib")]
            if name + "_write_kib" in vals:
                out[name] = (vals[k] * f_scale + vals[name + "_write_kib"] * w_scale) * 1024.0
    return out


def run_probes():
    """Ceilings measured on this device, right now, by the probe kernels of paper_2203_04071_amd/csrc/probes.hip."""
    import ctypes
    from paper_2203_04071_amd import build as hip_build
    if not os.path.exists(hip_build.PROBES_LIB):
        return None
    L = ctypes.CDLL(hip_build.PROBES_LIB)
    L.adapt_probe_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]

    def rate(which, iters):
        ms, units = ctypes.c_float(), ctypes.c_double()
        for _ in range(2):      # first run also brings the clocks up
            if L.adapt_probe_run(which, iters, ctypes.byref(ms), ctypes.byref(units)) != 0:
                raise SystemExit("bench.py: probe %d failed" % which)
        return units.value / (ms.value * 1e-3), ms.value

    cus = L.adapt_probe_cu_count()
    g16, _ = rate(0, 4000)
    g16g, _ = rate(1, 4000)
    b128, _ = rate(2, 1000)
    dma, _ = rate(3, 720)
    mfma, _ = rate(4, 2000)
    _, ms5 = rate(5, 720)
    return dict(cus=cus,
                lds_gather16_conflict_free_Tlookup_s=g16 / 1e12,
                lds_gather16_gaussian_row_Tlookup_s=g16g / 1e12,
                lds_read_b128_TB_s=b128 / 1e12,
                l2_to_lds_TB_s=dma / 1e12,
                mfma_i32_16x16x64_i8_Ginst_s=mfma / 1e9,
                quad_step_all_three_us=ms5 * 1e3 / 720,
                how="probe kernels run by this script before the timed region (16 waves per compute unit; best of 3 launches each)")


def probe_report():
    """--probe-report: every probe of the probes library, as one JSON line (units per second and clocks per 64-lane access
    for the LDS gathers; the figures behind the statements about gather cost in the recurrent step)."""
    import ctypes
    from paper_2203_04071_amd import build as hip_build
    if not os.path.exists(hip_build.PROBES_LIB):
        raise SystemExit("bench.py: %s is not built (python -c 'import __graft_entry__ as g; g.build()')" % hip_build.PROBES_LIB)
    L = ctypes.CDLL(hip_build.PROBES_LIB)
    L.adapt_probe_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    cus = L.adapt_probe_cu_count()
    names = {0: "gather of 2-byte entries, conflict-free addresses", 1: "gather of 2-byte entries, Gaussian codes in one 512-byte row (8 bits)",
             6: "gather of 2-byte entries, uniform codes in one 256-byte row (7 bits)",
             7: "as 6 with two copies of the row rotated by half the banks, lanes alternating",
             8: "gather of 1-byte entries, uniform codes in one 128-byte row", 9: "row held in registers, entries fetched with ds_bpermute",
             2: "16-byte reads in the quad kernel's pattern (bytes)", 3: "64 KB table copies L2 -> LDS, waited for one by one (bytes)",
             4: "v_mfma_i32_16x16x64_i8 (instructions)", 5: "copy + reads + matrix instructions of one quad step (steps x workgroups)"}
    iters = {0: 2000, 1: 2000, 6: 2000, 7: 2000, 8: 2000, 9: 2000, 2: 1000, 3: 720, 4: 2000, 5: 720}
    out = []
    for which in (0, 1, 6, 7, 8, 9, 2, 3, 4, 5):
        ms, units = ctypes.c_float(), ctypes.c_double()
        for _ in range(2):
            if L.adapt_probe_run(which, iters[which], ctypes.byref(ms), ctypes.byref(units)) != 0:
                raise SystemExit("bench.py: probe %d failed" % which)
        per_s = units.value / (ms.value * 1e-3)
        row = dict(probe=which, what=names[which], ms=round(ms.value, 4), units_per_s=per_s)
        if which in (0, 1, 6, 7, 8, 9):     # lookups: clocks one 64-lane gather occupies a compute unit's LDS, at 2.4 GHz
            row["clk_per_64_lane_gather"] = round(64.0 / (per_s / (cus * 2.4e9)), 2)
        out.append(row)
    print(json.dumps(dict(cus=cus, clock_ghz_assumed=2.4, probes=out)))


def elementwise_report(torch, B, elements):
    """--elementwise-report: the HBM-bound kernels of the path (range, quantiser, rescaling, histogram, fp32 glue) on a
    tensor far larger than the caches, each timed with events on the launch stream over back-to-back launches, beside a
    plain device-to-device copy of the same tensor timed the same way.  One JSON line: bytes per launch (what the
    operation has to read and write), GB/s, and that rate as a fraction of the copy's and of the published 8 TB/s."""
    n = int(elements)
    g = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn(n, device="cuda", generator=g)
    x2 = torch.randn(n, device="cuda", generator=g)
    y = torch.empty_like(x)
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    acc = torch.randint(-1 << 20, 1 << 20, (n,), dtype=torch.int32, device="cuda", generator=g)
    amax = torch.zeros(1, device="cuda")
    B.adapt_absmax_f32(x, amax_out=amax)
    torch.cuda.synchronize()
    a = float(amax.item())
    scale = a / 127.0
    counts = torch.zeros(2048, dtype=torch.int32, device="cuda")     # (accumulated into: 33 launches stay far below 2^32 per bin)
    chans = 64
    inner = n // (16 * chans)
    if 16 * chans * inner != n:
        raise SystemExit("bench.py: --elements must be a multiple of 1024")
    bias = torch.randn(chans, device="cuda", generator=g)
    ops = [
        ("copy (torch copy_, fp32 -> fp32)", 8 * n, lambda: y.copy_(x)),
        ("absmax", 4 * n, lambda: B.adapt_absmax_f32(x, amax_out=amax)),
        ("quantize fp32 -> int8", 5 * n, lambda: B.adapt_quantize_f32(x, scale, 8, out=q)),
        ("dequant int32 -> fp32 (+ bias)", 8 * n, lambda: B.adapt_dequant_i32(acc, 1e-3, 16, chans, inner, bias=bias, out=y)),
        ("relu", 8 * n, lambda: B.adapt_relu_f32(x, out=y)),
        ("add (residual)", 12 * n, lambda: B.adapt_add_f32(x, x2, out=y)),
        ("histogram of |x|, 2048 bins", 4 * n, lambda: B.adapt_histogram_abs_f32(x, a, 2048, counts=counts)),
    ]
    rows = []
    copy_rate = None
    for name, nbytes, fn in ops:
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        reps = 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best = None
        for _ in range(3):
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            best = ms if best is None or ms < best else best
        rate = nbytes / (best * 1e-3)
        if copy_rate is None:
            copy_rate = rate
        rows.append(dict(op=name, bytes_per_launch=nbytes, ms=round(best, 4), GB_s=round(rate / 1e9, 1),
                         frac_of_copy=round(rate / copy_rate, 3), frac_of_8TBs=round(rate / 8e12, 3)))
    print(json.dumps(dict(elements=n, note="events on torch's current stream, which is the stream these calls launch on; best of 3 blocks of 10 launches",
                          ops=rows)))


def _f(x):
    return np.float32(x)


def _graph_step(gnet, net, x, mode, many_small_launches):
    """A step of a network configuration is either one replay of the forward pass recorded into a HIP graph or the same
    kernels launched one by one.  Default: the graph where the pass is a chain of many small launches (ResNet-style CNN:
    34, recurrent layers: 200), launches one by one where it is a handful of kernels (measured: config 1 16 against 20 us,
    the separable block 52 against 57 us, the generator the same on most boxes and 6 % faster on one; a replay costs a
    few microseconds by itself).  --eager / --graph force one or the other."""
    if mode == "eager" or (mode is None and not many_small_launches):
        return lambda: net.forward(x)
    cap = gnet.Captured(net, x)
    return lambda: cap.replay()


def build_step(cfg_id, bits, torch, B, gnet, wl, eager=False, mode=None):
    """Returns (step_fn, core_fn, macs, workload_name, dtype) for a configuration.
    step_fn(): one pass of the whole path; core_fn(): only the dominant table-lookup call."""
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if cfg_id == 1:
        c = wl.config1()
        L = B.Lut(c["lut"], 8)
        A, W = dev(c["A"]), dev(c["W"])
        acc = torch.empty((64, 128), dtype=torch.int32, device="cuda")
        y = torch.empty((64, 128), dtype=torch.float32, device="cuda")

        pw = B.adapt_weights_pack_linear(L, W)      # weights are static: packed once, outside the timed steps

        def core():
            B.adapt_approx_linear_packed(pw, A, out=acc)

        class _Step:        # product + dequantise: two launches of a few microseconds, replayed as one HIP graph unless --eager
            def forward(self, a):
                B.adapt_approx_linear_packed(pw, a, out=acc)
                return B.adapt_dequant_i32(acc, c["scale"], 64, 128, 1, out=y)
        step = _graph_step(gnet, _Step(), A, mode, False)
        return step, core, 64 * 256 * 128, "config1: approx_linear 64x256x128, 8-bit table", (L, pw)
    if cfg_id == 2:
        c = wl.config2()
        L = B.Lut(c["lut"], 8)
        x, w = dev(c["x"]), dev(c["w"])
        s_x = gnet.calibrated_scale(x, 8)
        qw, s_w = gnet.quantize_weights(w, 8)
        qx = torch.empty(x.shape, dtype=torch.int8, device="cuda")
        acc = torch.empty((32, 64, 32, 32), dtype=torch.int32, device="cuda")
        y = torch.empty((32, 64, 32, 32), dtype=torch.float32, device="cuda")
        s_out = _f(s_x) * _f(s_w)
        B.adapt_quantize_f32(x, s_x, 8, out=qx)
        pw = B.adapt_weights_pack_conv2d(L, qw)      # weights are static: packed once, outside the timed steps

        # one fused call: the quantiser runs in the kernel that lays the input out for the product, the rescaling in
        # the product kernel (two launches; --eager times the four separate calls instead)
        def core():
            B.adapt_conv2d_layer_f32(pw, x, s_x, s_out, (1, 1), (1, 1), out=y)

        def step_separate():
            B.adapt_quantize_f32(x, s_x, 8, out=qx)
            B.adapt_approx_conv2d_packed(pw, qx, (1, 1), (1, 1), out=acc)
            B.adapt_dequant_i32(acc, s_out, 32, 64, 1024, out=y)

        # the product kernel alone, for the roofline: a second handle whose quantised, padded input copy is made once
        # (the chained-layer entry point runs only the product kernel when the copy is already in place)
        pk = B.adapt_weights_pack_conv2d(L, qw)
        yk = torch.empty_like(y)
        B.adapt_conv2d_chain_prepare(pk, 32, 32, 32, (1, 1), (1, 1))
        B.adapt_conv2d_layer_chain_f32(pk, x, s_x, s_out, yk, (1, 1), (1, 1))

        def kernel_only():
            B.adapt_conv2d_layer_chain_f32(pk, None, s_x, s_out, yk, (1, 1), (1, 1), in_shape=(32, 32, 32))

        core()
        kernel_only()
        torch.cuda.synchronize()
        if not torch.equal(y.view(torch.int32), yk.view(torch.int32)):
            raise SystemExit("bench.py: the product kernel on the prepared copy disagrees with the layer call")
        core.kernel_only = kernel_only
        core.keep = (pk, yk)

        step = step_separate if eager else core
        return step, core, wl.lut_macs_conv2d(32, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1), \
            "config2: approx_conv2d 3x3 s1 p1, batch 32, 64->64 ch, 32x32, 8-bit table", L
    if cfg_id == 3:
        c = wl.config3()
        net = gnet.ResNet20(c)
        x = dev(c["x"])
        net.forward(x)            # calibration pass (host reads), scales frozen afterwards
        step = _graph_step(gnet, net, x, mode, True)
        return step, None, gnet.lut_macs_resnet20(128), "config3: ResNet-20-style CNN, batch 128, 8-bit table", net
    if cfg_id == 4:
        c = wl.config4()
        net = gnet.LSTM(c)
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, mode, True)
        return step, None, gnet.lut_macs_lstm(100, 64, 512, 512), "config4: LSTM 512/512, seq 100, batch 64, 7-bit table", net
    if cfg_id == 5:
        c = wl.config5(bits=bits)
        net = gnet.DCGAN(c)
        z = dev(c["z"])
        net.forward(z)
        step = _graph_step(gnet, net, z, mode, False)
        return step, None, gnet.lut_macs_dcgan(256, c["plan"]), f"config5: DCGAN-style generator, batch 256, {bits}-bit table", net
    if cfg_id == 6:     # beyond the five baseline configurations: separable convolution block (Sec. III-B, eq. (1))
        c = wl.separable_workload(batch=32, cin=128, cout=128, hw=32)
        net = gnet.SeparableConv(c)
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, mode, False)
        macs = wl.lut_macs_conv2d(32, 128, 32, 32, 128, 3, 3, 1, 1, 1, 1, groups=128) + wl.lut_macs_conv2d(32, 128, 32, 32, 128, 1, 1, 1, 1, 0, 0)
        return step, None, macs, "extra: separable convolution 3x3 depthwise + 1x1, batch 32, 128->128 ch, 32x32, 8-bit table", net
    if cfg_id == 7:     # GRU layer at the size of the LSTM configuration (Sec. III-B "RNN Layer")
        c = wl.recurrent_workload("gru", seq=100, batch=64, isz=512, hsz=512, bits=7)
        net = gnet.Recurrent(c, "gru")
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, mode, True)
        return step, None, 100 * 64 * 3 * 512 * (512 + 512), "extra: GRU 512/512, seq 100, batch 64, 7-bit table", net
    if cfg_id in (8, 9):    # the layer of configuration 2 with 12-bit operands: table in device memory (8) / Mitchell function (9)
        c = wl.config2()
        x = dev(c["x"])
        w = dev(c["w"])
        s_x = gnet.calibrated_scale(x, 12)
        s_w = gnet.calibrated_scale(w, 12)
        qw = B.adapt_quantize_i16_f32(w, s_w, 12)
        qx = torch.empty(x.shape, dtype=torch.int16, device="cuda")
        acc = torch.empty((32, 64, 32, 32), dtype=torch.int32, device="cuda")
        y = torch.empty((32, 64, 32, 32), dtype=torch.float32, device="cuda")
        s_out = _f(s_x) * _f(s_w)
        L = B.Lut16(12, table=wl.make_lut(12)) if cfg_id == 8 else None

        def core():
            if cfg_id == 8:
                B.adapt_approx_conv2d_i16(L, qx, qw, (1, 1), (1, 1), out=acc)
            else:
                B.adapt_approx_conv2d_func_i16(B.FUNC_MITCHELL, 0, 12, qx, qw, (1, 1), (1, 1), out=acc)

        def step():
            B.adapt_quantize_i16_f32(x, s_x, 12, out=qx)
            core()
            B.adapt_dequant_i32(acc, s_out, 32, 64, 1024, out=y)
        name = ("extra: approx_conv2d 3x3 s1 p1, batch 32, 64->64 ch, 32x32, 12-bit " +
                ("table in device memory" if cfg_id == 8 else "Mitchell multiplier as a function"))
        return step, core, wl.lut_macs_conv2d(32, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1), name, L
    if cfg_id == 10:    # retraining (Sec. III-A): straight-through backward pass of the recurrent configuration's input projection
        M, K, N = 6400, 512, 2048
        rng = np.random.default_rng(1234 + 10)
        x = dev(rng.standard_normal((M, K)).astype(np.float32))
        w = dev((rng.standard_normal((N, K)) * 0.1).astype(np.float32))
        dy = dev(rng.standard_normal((M, N)).astype(np.float32))
        s_x = gnet.calibrated_scale(x, 7)
        s_w = gnet.calibrated_scale(w, 7)
        outs = [torch.empty((M, K), dtype=torch.float32, device="cuda"), torch.empty((N, K), dtype=torch.float32, device="cuda"),
                torch.empty((N,), dtype=torch.float32, device="cuda")]

        def core():
            B.adapt_ste_linear_backward_f32(dy, x, w, s_x, s_w, 7, out=outs)
        name = "extra: straight-through backward pass of a linear layer, 6400 x 512 -> 2048, 7-bit operands (dx, dw, db)"
        return core, core, 2 * M * K * N, name, outs
    if cfg_id == 11:    # retraining: straight-through backward pass of the headline convolution layer (configuration 2's shape)
        c = wl.config2()
        x = dev(c["x"]); w = dev(c["w"])
        dy = dev(np.random.default_rng(1234 + 11).standard_normal((32, 64, 32, 32)).astype(np.float32))
        s_x = gnet.calibrated_scale(x, 8)
        s_w = gnet.calibrated_scale(w, 8)
        ws = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")

        def core():
            B.adapt_ste_conv2d_backward_f32(dy, x, w, (1, 1), (1, 1), (1, 1), s_x, s_w, 8, workspace=ws)
        name = "extra: straight-through backward pass of the 3x3 convolution layer, batch 32, 64->64 ch, 32x32, 8-bit operands (dx, dw, db)"
        return core, core, 2 * 32768 * 576 * 64, name, ws
    raise SystemExit(f"unknown config {cfg_id}")


def cpu_baseline(cfg_id, bits, wl):
    """The parity oracle as it stands, timed on this host's cores, on a bounded sample."""
    import oracle as orc
    from oracle import networks as onet
    th = orc.host_threads()
    if cfg_id == 1:
        c = wl.config1()
        reps, macs = 20, 64 * 256 * 128
        t0 = time.perf_counter()
        for _ in range(reps):
            acc = orc.approx_linear(c["lut"], 8, c["A"], c["W"], threads=th)
            orc.dequant(acc, c["scale"], 64, 128, 1)
        dt = (time.perf_counter() - t0) / reps
        return dict(value=macs / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample=f"full config-1 layer, mean of {reps} passes")
    if cfg_id == 2:
        c = wl.config2()
        s_x = orc.scale_from_amax(orc.absmax(c["x"]), 8)
        s_w = orc.scale_from_amax(orc.absmax(c["w"]), 8)
        qw = orc.quantize(c["w"], s_w, 8)
        macs = wl.lut_macs_conv2d(32, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1)
        best = 1e30
        reps = 5
        for _ in range(reps):
            t0 = time.perf_counter()
            qx = orc.quantize(c["x"], s_x, 8)
            acc = orc.approx_conv2d(c["lut"], 8, qx, qw, (1, 1), (1, 1), threads=th)
            orc.dequant(acc, _f(s_x) * _f(s_w), 32, 64, 1024)
            best = min(best, time.perf_counter() - t0)
        return dict(value=macs / best, unit="LUT-MAC/s", cores=th, kind="oracle",
                    sample=f"full config-2 step (32 images: quantise + conv + dequantise), best of {reps} passes")
    if cfg_id == 3:
        c = wl.config3(batch=32)
        t0 = time.perf_counter()
        onet.resnet20(c, threads=th)
        dt = time.perf_counter() - t0
        macs = 40551040 * 32
        return dict(value=macs / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample="32 of 128 images, one pass incl. calibration")
    if cfg_id == 4:
        c = wl.config4()
        t0 = time.perf_counter()
        onet.lstm(c, threads=th, steps=10)
        dt = time.perf_counter() - t0
        return dict(value=134217728 * 10 / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample="first 10 of 100 time steps")
    if cfg_id == 6:
        c = wl.separable_workload(batch=8, cin=128, cout=128, hw=32)
        t0 = time.perf_counter()
        onet.separable_conv(c, threads=th)
        dt = time.perf_counter() - t0
        macs = wl.lut_macs_conv2d(8, 128, 32, 32, 128, 3, 3, 1, 1, 1, 1, groups=128) + wl.lut_macs_conv2d(8, 128, 32, 32, 128, 1, 1, 1, 1, 0, 0)
        return dict(value=macs / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample="8 of 32 images, one pass incl. calibration")
    if cfg_id == 7:
        c = wl.recurrent_workload("gru", seq=100, batch=64, isz=512, hsz=512, bits=7)
        t0 = time.perf_counter()
        onet.gru(c, threads=th, steps=10)
        dt = time.perf_counter() - t0
        return dict(value=64 * 3 * 512 * 1024 * 10 / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample="first 10 of 100 time steps")
    if cfg_id in (8, 9):
        c = wl.config2()
        s_x = orc.scale_from_amax(orc.absmax(c["x"]), 12)
        s_w = orc.scale_from_amax(orc.absmax(c["w"]), 12)
        qw = orc.quantize_i16(c["w"], s_w, 12)
        lut = wl.make_lut(12) if cfg_id == 8 else None
        t0 = time.perf_counter()
        qx = orc.quantize_i16(c["x"][:8], s_x, 12)
        acc = orc.approx_conv2d_i16(12, qx, qw, lut=lut, func=None if cfg_id == 8 else (orc.FUNC_MITCHELL, 0), pad=(1, 1), threads=th)
        orc.dequant(acc, _f(s_x) * _f(s_w), 8, 64, 1024)
        dt = time.perf_counter() - t0
        return dict(value=wl.lut_macs_conv2d(8, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1) / dt, unit="LUT-MAC/s", cores=th, kind="oracle",
                    sample="8 of 32 images, one pass")
    if cfg_id == 11:
        from oracle import ste
        c = wl.config2()
        x = c["x"][:8]
        dy = np.random.default_rng(1234 + 11).standard_normal((8, 64, 32, 32)).astype(np.float32)
        s_x = orc.scale_from_amax(orc.absmax(c["x"]), 8)
        s_w = orc.scale_from_amax(orc.absmax(c["w"]), 8)
        t0 = time.perf_counter()
        ste.ste_conv2d_backward(dy, x, c["w"], (1, 1), (1, 1), (1, 1), s_x, s_w, 8)
        dt = time.perf_counter() - t0
        return dict(value=4.0 * 8 * 1024 * 576 * 64 / dt, unit="FLOP/s", cores=th, kind="oracle",
                    sample="8 of 32 images, one pass (fp64; tap by tap with numpy's einsum)")
    if cfg_id == 10:
        from oracle import ste
        M, K, N = 1600, 512, 2048
        rng = np.random.default_rng(1234 + 10)
        x = rng.standard_normal((M, K)).astype(np.float32)
        w = (rng.standard_normal((N, K)) * 0.1).astype(np.float32)
        dy = rng.standard_normal((M, N)).astype(np.float32)
        s_x = orc.scale_from_amax(orc.absmax(x), 7)
        s_w = orc.scale_from_amax(orc.absmax(w), 7)
        t0 = time.perf_counter()
        ste.ste_linear_backward(dy, x, w, s_x, s_w, 7)
        dt = time.perf_counter() - t0
        return dict(value=4.0 * M * K * N / dt, unit="FLOP/s", cores=th, kind="oracle",
                    sample="1600 of 6400 rows, one pass (fp64; its two matrix products are numpy's)")
    c = wl.config5(bits=bits, batch=32)
    t0 = time.perf_counter()
    onet.dcgan(c, threads=th)
    dt = time.perf_counter() - t0
    return dict(value=104628224 * 32 / dt, unit="LUT-MAC/s", cores=th, kind="oracle", sample="32 of 256 latent vectors, one pass incl. calibration")


def network_roofline(cfg_id, bits, macs, ms_per_step, ceilings, model_peak, gnet):
    """A whole network step priced against the measured ceilings: the time its lookups need at the rate of the resource
    that bounds the kernel they run on (16-byte LDS reads for the derived-table kernels: 2 bytes per lookup; 16-bit LDS
    gathers for the whole-table kernel: one per lookup), divided by the measured step time."""
    if not ceilings or cfg_id not in (3, 4, 5, 6, 7):
        return None
    lds = ceilings["lds_read_b128_TB_s"] * 1e12
    g16 = ceilings["lds_gather16_conflict_free_Tlookup_s"] * 1e12
    if cfg_id == 4:
        rec = 100 * 64 * 512 * 2048          # hidden-state products: one launch per time step on the whole-table kernel
        proj = macs - rec                    # input products of all steps: one launch of the quad kernel
        t = rec / g16 + 2.0 * proj / lds
        dom, bound = "lut_rows_kernel (recurrent step: product + cell, 100 launches)", "lds_gather16 (recurrence) + lds_read (input products)"
    elif cfg_id == 7:
        rec = 100 * 64 * 512 * 1536
        t = rec / g16 + 2.0 * (macs - rec) / lds
        dom, bound = "lut_rows_kernel (recurrent step: product + cell, 100 launches)", "lds_gather16 (recurrence) + lds_read (input products)"
    else:
        t = 2.0 * macs / lds
        dom = {3: "lut_quad_kernel (stride-1 layers; the 32- and 64-channel ones in slices + reduce_partials_kernel); 19 layers of 13 - 23 us",
               5: "lut_quad_kernel<%d, 8, true>" % (2 if bits == 8 else 1),
               6: "lut_grouped_tiled_kernel + lut_quad_kernel"}[cfg_id]
        bound = "lds_read"
    return dict(bound=bound, achieved=macs / (ms_per_step * 1e-3) / 1e12, peak=macs / t / 1e12, unit="Tlookup/s", frac=t / (ms_per_step * 1e-3),
                traffic=None, bound_us=t * 1e6, dominant_kernel=dom, covers="the whole network step (every kernel, launch gaps included)",
                peak_source="what the step's lookups cost at the LDS rates measured by the probe kernels in this run", ceilings=ceilings)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="1-5: the baseline configurations (default 2, the one the metric is quoted on); "
                    "6: separable convolution block, 7: GRU layer, 8 / 9: the layer of 2 with 12-bit operands, table / function form, "
                    "10 / 11: straight-through backward pass of a linear / convolution layer "
                    "(rows beyond the baseline, not bench lines of record)")
    ap.add_argument("--bits", type=int, default=8, help="table bits for config 5 (6 or 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the ceiling probes (roofline then falls back to model figures or is omitted)")
    ap.add_argument("--no-others", action="store_true", help="default run: do not time the other baseline configurations after the headline one")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps for each of the other configurations of the default run")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="untimed steps for this long before the warm-up steps, so that the device clocks have settled (0: none)")
    ap.add_argument("--eager", action="store_true", help="network configurations: launch kernel by kernel (default for configs 1, 5, 6); "
                    "config 2: the separate calls instead of the fused layer call")
    ap.add_argument("--graph", action="store_true", help="network configurations: replay a HIP graph (default for configs 3, 4, 7)")
    ap.add_argument("--probe-report", action="store_true", help="run every ceiling probe and print their rates as one JSON line; nothing else")
    ap.add_argument("--elementwise-report", action="store_true",
                    help="time the HBM-bound element-wise kernels on a large tensor beside a plain copy and print one JSON line; nothing else")
    ap.add_argument("--elements", type=float, default=float(1 << 26), help="tensor size for --elementwise-report (default 64 Mi elements)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three plain 64 MiB device-to-device copies (what FETCH_SIZE / WRITE_SIZE are scaled by)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc (reported as roofline.traffic)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (pure batch sharding would need no exchange step). "
                         "Run with --gpus 1.")

    import torch
    from paper_2203_04071_amd import binding as B, networks as gnet, workloads as wl
    if not torch.cuda.is_available():
        raise SystemExit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    B.load()
    torch.cuda.set_device(0)
    if args.probe_report:
        probe_report()
        return
    if args.elementwise_report:
        elementwise_report(torch, B, args.elements)
        return
    if args.copy_calibration:
        a = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 64 << 20, "copies": 3}))
        return
    # ceilings of this device, measured now (headline and network configurations price their kernels against them)
    ceilings = run_probes() if args.config <= 7 and not args.no_probes else None
    step, core, macs, name, _keep = build_step(args.config, args.bits, torch, B, gnet, wl, args.eager, "eager" if args.eager else ("graph" if args.graph else None))

    def timed(step_fn, steps, warmup, prewarm_ms):
        # bring the device to its running clocks before anything is measured (a cold GPU runs the first tens of
        # milliseconds slower; the W warm-up steps of the small configurations are over in well under a millisecond)
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < prewarm_ms * 1e-3:
            for _ in range(20):
                step_fn()
            torch.cuda.synchronize()
        for _ in range(warmup):
            step_fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step_fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_per_step = timed(step, args.steps, args.warmup, args.prewarm_ms)

    # dominant kernel: HIP events on the launch stream around the table-lookup call
    roof = None
    cus = B.adapt_device_cu_count()
    model_peak = cus * LDS_LANES_PER_CLK_PER_CU * MODEL_CLOCK_GHZ * 1e9
    traffic_by_kernel = read_traffic()
    traffic = args.traffic_bytes

    def lookup_context(rate):
        """The metric's own model: lookups per second against one 2-byte lookup per bank-lane and clock."""
        d = dict(achieved_Tlookup_s=rate / 1e12, model_peak_Tlookup_s=model_peak / 1e12, frac_of_model=rate / model_peak,
                 model=f"{cus} CUs x {LDS_LANES_PER_CLK_PER_CU} LDS bank-lanes/clk x {MODEL_CLOCK_GHZ} GHz; 1 lookup (2 B) per LUT-MAC")
        if ceilings:
            g = ceilings["lds_gather16_conflict_free_Tlookup_s"] * 1e12
            d.update(measured_conflict_free_gather_Tlookup_s=g / 1e12, frac_of_measured_gather=rate / g,
                     note="a kernel on derived tables reads 16 bytes (8 entries) per LDS lane-access, so these two fractions are not "
                          "bounded by 1 for it; its ceilings are the resources in roofline.resource_us")
        return d

    if core is not None:
        # back-to-back launches between one pair of events per block, so the queue stays full and the figure is the
        # device time of the call's kernels, comparable with a kernel trace
        def event_ms(fn):
            blocks, per = 5, max(1, args.steps // 5)
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(blocks)]
            torch.cuda.synchronize()
            for a, b in evs:
                a.record()
                for _ in range(per):
                    fn()
                b.record()
            torch.cuda.synchronize()
            return np.array([a.elapsed_time(b) / per for a, b in evs])

        call_ms = event_ms(core)
        kernel_only = getattr(core, "kernel_only", None)
        kms = event_ms(kernel_only) if kernel_only is not None else call_ms
        k_avg = float(kms.mean())
        achieved = macs / (k_avg * 1e-3)
        if args.config == 2 and ceilings:
            # The product kernel of the headline layer (lut_quad_kernel), priced resource by resource: what one launch
            # needs of each, divided by what the probes measured for it a moment ago.  The largest of these times is the
            # bound; frac = that time / the kernel's measured time.
            kern, rpw, ksplit, steps_k, wgs = B.adapt_plan_packed(1, 8, 0, 64, 64, 3, 3, 1, 32768, 32, 1)
            if kern != 3:
                raise SystemExit("bench.py: the headline layer is not planned on the quad kernel")
            table_bytes = 256 << 8
            lds_bytes = 2.0 * macs                                          # one 16-byte read per 8 lookups
            fill_bytes = float(wgs) * (steps_k / ksplit) * (table_bytes + rpw * 16)  # tables into LDS + activations into registers, per step
            mfma_insts = macs / 512.0                                       # one matrix instruction per 64 reads
            hbm_bytes = 32 * 34 * 34 * 64 + 8 * steps_k * table_bytes + 4.0 * 32 * 64 * 32 * 32      # padded copy + tables + fp32 output
            res_us = dict(lds_read=lds_bytes / (ceilings["lds_read_b128_TB_s"] * 1e12) * 1e6,
                          l2_to_cu_fill=fill_bytes / (ceilings["l2_to_lds_TB_s"] * 1e12) * 1e6,
                          mfma=mfma_insts / (ceilings["mfma_i32_16x16x64_i8_Ginst_s"] * 1e9) * 1e6,
                          hbm=hbm_bytes / HBM_PEAK_BYTES_PER_S * 1e6)
            bound = max(res_us, key=res_us.get)
            amount, peak_v, unit = {"lds_read": (lds_bytes, ceilings["lds_read_b128_TB_s"], "TB/s"),
                                    "l2_to_cu_fill": (fill_bytes, ceilings["l2_to_lds_TB_s"], "TB/s"),
                                    "mfma": (mfma_insts * 32768, ceilings["mfma_i32_16x16x64_i8_Ginst_s"] * 1e9 * 32768 / 1e12, "TOP/s"),
                                    "hbm": (hbm_bytes, HBM_PEAK_BYTES_PER_S / 1e12, "TB/s")}[bound]
            if traffic is None:
                traffic = traffic_by_kernel.get("lut_quad_kernel")
            roof = dict(bound=bound, achieved=amount / (k_avg * 1e-3) / 1e12, peak=peak_v, unit=unit, frac=res_us[bound] / (k_avg * 1e3),
                        traffic=traffic, traffic_source=os.path.relpath(TRAFFIC_FILE, ROOT) if traffic is not None and args.traffic_bytes is None else None,
                        kernel="lut_quad_kernel<4, %d, false>" % (rpw // 256), kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()),
                        call_ms_avg=float(call_ms.mean()), call_traffic=(traffic + traffic_by_kernel["pad_channels_last"]) if traffic is not None and "pad_channels_last" in traffic_by_kernel else None,
                        covers="the product kernel alone, launched on an input copy made beforehand; call_ms_avg adds the call's quantise-and-copy kernel",
                        resource_us=res_us, algorithmic=dict(lds_bytes=lds_bytes, l2_to_cu_fill_bytes=fill_bytes, mfma_instructions=mfma_insts, hbm_bytes=hbm_bytes,
                                                             workgroups=wgs, steps=steps_k, rows_per_workgroup=rpw),
                        all_three_together_us=ceilings["quad_step_all_three_us"] * steps_k / ksplit * ((wgs + cus - 1) // cus),
                        peak_source="measured by the probe kernels in this run (roofline.ceilings)", ceilings=ceilings,
                        lookups=lookup_context(achieved))
        elif args.config in (10, 11):
            # two dense fp32 contractions (macs counts the multiply-adds of both): the matrix pipe's fp32 rate
            roof = dict(bound="mfma", achieved=2 * achieved / 1e12, peak=157.3, unit="TFLOP/s", frac=2 * achieved / 157.3e12, traffic=None,
                        kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()), covers="every kernel of the call (products, bias gradient; convolution: also the unfolding and gathering kernels)",
                        peak_model="published dense fp32 matrix rate of MI355X")
        elif args.config == 8:
            # a table beyond LDS is gathered through the vector memory path: 4 lane addresses per clock per compute unit
            gpeak = cus * GATHER_LANES_PER_CLK_PER_CU * MODEL_CLOCK_GHZ * 1e9
            roof = dict(bound="l1-gather", achieved=achieved / 1e12, peak=gpeak / 1e12, unit="Tlookup/s", frac=achieved / gpeak, traffic=traffic,
                        kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()),
                        peak_model=f"{cus} CUs x {GATHER_LANES_PER_CLK_PER_CU} gathered lanes/clk x {MODEL_CLOCK_GHZ} GHz; 1 lookup (4 B from device memory) per LUT-MAC")
        elif args.config == 9:
            # the multiplier as a function: vector integer operations, 64 lanes per clock per compute unit
            apeak = cus * 64 * MODEL_CLOCK_GHZ * 1e9 / MITCHELL_OPS_PER_MAC
            roof = dict(bound="alu", achieved=achieved / 1e12, peak=apeak / 1e12, unit="TMAC/s", frac=achieved / apeak, traffic=traffic,
                        kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()),
                        peak_model=f"{cus} CUs x 64 lanes/clk x {MODEL_CLOCK_GHZ} GHz / {MITCHELL_OPS_PER_MAC} vector instructions per Mitchell multiply-accumulate")
        else:
            # whole-table kernel (configuration 1 and other short products): one 16-bit LDS gather per lookup
            g = (ceilings["lds_gather16_conflict_free_Tlookup_s"] * 1e12) if ceilings else model_peak
            roof = dict(bound="lds_gather16", achieved=achieved / 1e12, peak=g / 1e12, unit="Tlookup/s", frac=achieved / g, traffic=traffic,
                        kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()), covers="every kernel of the table-lookup call",
                        peak_source="conflict-free 16-bit LDS gathers measured by the probe kernel in this run" if ceilings else "model",
                        ceilings=ceilings, lookups=lookup_context(achieved))
    else:
        roof = network_roofline(args.config, args.bits, macs, ms_per_step, ceilings, model_peak, gnet)
        if roof is not None:
            roof["lookups"] = lookup_context(macs / (ms_per_step * 1e-3))

    # the other baseline configurations, after the headline measurement (default run only)
    others = None
    if args.config == 2 and not args.no_others:
        others = []
        del step, core, _keep
        torch.cuda.empty_cache()
        for cfg, bits in ((1, 8), (3, 8), (4, 7), (5, 6), (5, 8)):
            st, co, m, nm, keep = build_step(cfg, bits, torch, B, gnet, wl, False)
            ms = timed(st, args.other_steps, 3, 100.0)
            entry = dict(workload=nm, lut_macs_per_step=m, steps=args.other_steps, ms_per_step=ms, value=m / (ms * 1e-3), unit="LUT-MAC/s")
            if co is not None:
                g = ceilings["lds_gather16_conflict_free_Tlookup_s"] * 1e12 if ceilings else model_peak
                entry.update(dominant_kernel="lut_rows_kernel (whole table in LDS)", bound="lds_gather16", frac=m / (ms * 1e-3) / g)
            else:
                r = network_roofline(cfg, bits, m, ms, ceilings, model_peak, gnet)
                if r:
                    entry.update(dominant_kernel=r["dominant_kernel"], bound=r["bound"], frac=r["frac"], bound_us=r["bound_us"])
            others.append(entry)
            del st, co, keep
            torch.cuda.empty_cache()

    out = {
        "metric": ("approximate MACs/sec (LUT-MAC/s), whole step: quantise + table-lookup layer(s) + dequantise" if args.config not in (10, 11) else
                   "fp32 FLOP/s of the two gradient contractions (fake quantisation and clip masks included in the time)"),
        "value": macs / (ms_per_step * 1e-3) * (2 if args.config in (10, 11) else 1),
        "unit": "LUT-MAC/s" if args.config not in (10, 11) else "FLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("int8 operands, int16 table, int32 accumulate, fp32 scale" if args.config < 8 else
                  "f32" if args.config in (10, 11) else
                  "int16 operands (12-bit), int32 table or function, int32 accumulate, fp32 scale"),
        "data": "synthetic (seeded)", "prewarm_ms": args.prewarm_ms,
        "config": {"workload": name, ("lut_macs_per_step" if args.config not in (10, 11) else "multiply_adds_per_step"): macs},
        "roofline": roof,
    }
    if others is not None:
        out["others"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.bits, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
