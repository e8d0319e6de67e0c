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

LDS_LANES_PER_CLK_PER_CU = 32      # 32 banks x 4 B: one 16-bit gather lane per bank per clock
MODEL_CLOCK_GHZ = 2.4
GATHER_LANES_PER_CLK_PER_CU = 4    # vector memory path: one 64-lane gather instruction per 16 clocks
MITCHELL_OPS_PER_MAC = 15          # vector instructions per multiply-accumulate counted in the compiled function-form kernel (484 per 32)
MODEL_CUS = 256

# HBM bytes per launch of the dominant call, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, each
# scaled by what the same counter reads for a plain 64 MiB copy (--copy-calibration); figures and commands are in
# profiles/lut_lines_wide_config2.md.  Keyed by config number; None = not measured.
MEASURED_TRAFFIC_BYTES = {2: (18576 * 2.0 + 8192 * 1.0 + 4646 * 2.0 + 2312 * 1.0) * 1024}
# the product kernel alone (lut_lines_wide_kernel<4> at configuration 2), same runs
MEASURED_KERNEL_TRAFFIC_BYTES = {2: (18576 * 2.0 + 8192 * 1.0) * 1024}
# clocks the matrix pipe of a SIMD is busy per v_mfma_i32_16x16x64_i8 (SQ_VALU_MFMA_BUSY_CYCLES / SQ_INSTS_VALU_MFMA_I8 of
# that kernel, profiles/lut_lines_wide_config2.md)
MFMA_16X16X64_CLOCKS = 16


def _f(x):
    return np.float32(x)


def _graph_step(gnet, net, x, eager):
    """The network configurations are chains of many small launches: one step = one replay of the forward pass recorded
    into a HIP graph (same kernels, same order); --eager launches them one by one instead."""
    if eager:
        return lambda: net.forward(x)
    cap = gnet.Captured(net, x)
    return lambda: cap.replay()


def build_step(cfg_id, bits, torch, B, gnet, wl, eager=False):
    """Returns (step_fn, core_fn, macs, workload_name, dtype) for a configuration.
    step_fn(): one pass of the whole path; core_fn(): only the dominant table-lookup call."""
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if cfg_id == 1:
        c = wl.config1()
        L = B.Lut(c["lut"], 8)
        A, W = dev(c["A"]), dev(c["W"])
        acc = torch.empty((64, 128), dtype=torch.int32, device="cuda")
        y = torch.empty((64, 128), dtype=torch.float32, device="cuda")

        def core():
            B.adapt_approx_linear(L, A, W, out=acc)

        def step():
            core()
            B.adapt_dequant_i32(acc, c["scale"], 64, 128, 1, out=y)
        return step, core, 64 * 256 * 128, "config1: approx_linear 64x256x128, 8-bit table", L
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
        step = _graph_step(gnet, net, x, eager)
        return step, None, gnet.lut_macs_resnet20(128), "config3: ResNet-20-style CNN, batch 128, 8-bit table", net
    if cfg_id == 4:
        c = wl.config4()
        net = gnet.LSTM(c)
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, eager)
        return step, None, gnet.lut_macs_lstm(100, 64, 512, 512), "config4: LSTM 512/512, seq 100, batch 64, 7-bit table", net
    if cfg_id == 5:
        c = wl.config5(bits=bits)
        net = gnet.DCGAN(c)
        z = dev(c["z"])
        net.forward(z)
        step = _graph_step(gnet, net, z, eager)
        return step, None, gnet.lut_macs_dcgan(256, c["plan"]), f"config5: DCGAN-style generator, batch 256, {bits}-bit table", net
    if cfg_id == 6:     # beyond the five baseline configurations: separable convolution block (Sec. III-B, eq. (1))
        c = wl.separable_workload(batch=32, cin=128, cout=128, hw=32)
        net = gnet.SeparableConv(c)
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, eager)
        macs = wl.lut_macs_conv2d(32, 128, 32, 32, 128, 3, 3, 1, 1, 1, 1, groups=128) + wl.lut_macs_conv2d(32, 128, 32, 32, 128, 1, 1, 1, 1, 0, 0)
        return step, None, macs, "extra: separable convolution 3x3 depthwise + 1x1, batch 32, 128->128 ch, 32x32, 8-bit table", net
    if cfg_id == 7:     # GRU layer at the size of the LSTM configuration (Sec. III-B "RNN Layer")
        c = wl.recurrent_workload("gru", seq=100, batch=64, isz=512, hsz=512, bits=7)
        net = gnet.Recurrent(c, "gru")
        x = dev(c["x"])
        net.forward(x)
        step = _graph_step(gnet, net, x, eager)
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
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="untimed steps for this long before the warm-up steps, so that the device clocks have settled (0: none)")
    ap.add_argument("--eager", action="store_true", help="network configurations: launch kernel by kernel instead of replaying a HIP graph")
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
    if args.copy_calibration:
        a = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 64 << 20, "copies": 3}))
        return
    step, core, macs, name, _keep = build_step(args.config, args.bits, torch, B, gnet, wl, args.eager)

    # bring the device to its running clocks before anything is measured (a cold GPU runs the first tens of
    # milliseconds slower; the W warm-up steps of the small configurations are over in well under a millisecond)
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < args.prewarm_ms * 1e-3:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps

    # dominant kernel: HIP events on the launch stream around the table-lookup call
    roof = None
    cus = B.adapt_device_cu_count()
    traffic = args.traffic_bytes if args.traffic_bytes is not None else MEASURED_TRAFFIC_BYTES.get(args.config)
    peak = cus * LDS_LANES_PER_CLK_PER_CU * MODEL_CLOCK_GHZ * 1e9
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
        if kernel_only is not None:
            # the dominant kernel by itself (launched on an input copy made beforehand): the duration a kernel trace
            # lists for it; the call's other kernel (quantise + copy) is in call_ms_avg
            kms = event_ms(kernel_only)
            covers = "the product kernel alone (lut_lines_wide_kernel); call_ms_avg adds the call's quantise-and-copy kernel"
            if args.traffic_bytes is None:
                traffic = MEASURED_KERNEL_TRAFFIC_BYTES.get(args.config)
            # second bound of the same kernel: the pipe that widens and adds the entries.  With a table whose range fits
            # the digit form (this one does) that is the matrix pipe: two v_mfma_i32_16x16x64_i8 of 16 clocks per 512
            # lookups of a wave, four SIMDs per compute unit
            pipe_peak = cus * 4 * 512 / (2 * MFMA_16X16X64_CLOCKS) * MODEL_CLOCK_GHZ * 1e9
            extra_bound = dict(pipe_bound="mfma (int8)", pipe_peak=pipe_peak / 1e12,
                               pipe_frac=macs / (float(kms.mean()) * 1e-3) / pipe_peak,
                               pipe_model=f"{cus} CUs x 4 SIMDs x 512 lookups per 2 v_mfma_i32_16x16x64_i8 of "
                                          f"{MFMA_16X16X64_CLOCKS} clocks x {MODEL_CLOCK_GHZ} GHz")
        else:
            kms = call_ms
            covers = "every kernel of the table-lookup call"
            extra_bound = {}
        k_avg = float(kms.mean())
        achieved = macs / (k_avg * 1e-3)
        roof = dict(bound="lds", achieved=achieved / 1e12, peak=peak / 1e12, unit="Tlookup/s", frac=achieved / peak,
                    traffic=traffic, kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()),
                    call_ms_avg=float(call_ms.mean()), call_frac=macs / (float(call_ms.mean()) * 1e-3) / peak,
                    call_traffic=MEASURED_TRAFFIC_BYTES.get(args.config), covers=covers, **extra_bound,
                    peak_model=f"{cus} CUs x {LDS_LANES_PER_CLK_PER_CU} LDS bank-lanes/clk x {MODEL_CLOCK_GHZ} GHz; "
                               "1 lookup (2 B) per LUT-MAC")
        if args.config == 8:
            # a table beyond LDS is gathered through the vector memory path: 4 lane addresses per clock per compute unit
            gpeak = cus * GATHER_LANES_PER_CLK_PER_CU * MODEL_CLOCK_GHZ * 1e9
            roof.update(bound="l1-gather", peak=gpeak / 1e12, frac=achieved / gpeak,
                        peak_model=f"{cus} CUs x {GATHER_LANES_PER_CLK_PER_CU} gathered lanes/clk x {MODEL_CLOCK_GHZ} GHz; "
                                   "1 lookup (4 B from device memory) per LUT-MAC")
        if args.config in (10, 11):
            # two dense fp32 contractions (macs counts the multiply-adds of both): the matrix pipe's fp32 rate
            roof = dict(bound="mfma", achieved=2 * achieved / 1e12, peak=157.3, unit="TFLOP/s", frac=2 * achieved / 157.3e12, traffic=None,
                        kernel_ms_avg=k_avg, kernel_ms_min=float(kms.min()), covers="every kernel of the call (products, bias gradient; convolution: also the unfolding and gathering kernels)",
                        peak_model="published dense fp32 matrix rate of MI355X")
        if args.config == 9:
            # the multiplier as a function: vector integer operations, 64 lanes per clock per compute unit
            apeak = cus * 64 * MODEL_CLOCK_GHZ * 1e9 / MITCHELL_OPS_PER_MAC
            roof.update(bound="alu", peak=apeak / 1e12, unit="TMAC/s", frac=achieved / apeak,
                        peak_model=f"{cus} CUs x 64 lanes/clk x {MODEL_CLOCK_GHZ} GHz / {MITCHELL_OPS_PER_MAC} vector "
                                   "instructions per Mitchell multiply-accumulate")
    else:
        achieved = macs / (ms_per_step * 1e-3)
        roof = dict(bound="lds", achieved=achieved / 1e12, peak=peak / 1e12, unit="Tlookup/s", frac=achieved / peak,
                    traffic=traffic, note="whole network step (all kernels) against the LDS lookup peak")

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
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.bits, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
