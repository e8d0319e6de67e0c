"""Network-shaped workloads (CNN, LSTM, GAN families of Sec. V, Table I) as sequences of C-ABI
calls.  Every tensor operation is a library kernel; Python only orders the calls and holds the
per-layer scales (plain floats) that max-abs calibration produced.

Calibration (Sec. III-A, "max absolute number" scale) is progressive: the scale of a layer's
input is the max-abs of the fp32 tensor that the already-approximate earlier layers produce on
the calibration batch.  It needs one device->host read per layer and is therefore done once;
`scales=` replays a calibrated network without any synchronisation.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .workloads import resnet20_plan


def _f(x):
    return np.float32(x)


def scale_from_amax(amax: float, bits: int) -> np.float32:
    q = _f((1 << (bits - 1)) - 1)
    a = _f(amax)
    return _f(1.0) if not (a > 0) else a / q


def calibrated_scale(x, bits) -> np.float32:
    return scale_from_amax(B.adapt_absmax_f32(x).item(), bits)


def quantize_weights(w, bits):
    s = calibrated_scale(w, bits)
    return B.adapt_quantize_f32(w, s, bits), s


class Captured:
    """One forward pass of a calibrated network recorded into a HIP graph and replayed as a single launch.

    The networks are launch-bound chains of small kernels; a graph removes the per-launch host cost.  Recording needs
    a pass that neither allocates through the library nor reads anything back: scales must already be frozen and every
    packed-weights handle must have run once at this input size (its workspace is then large enough).  The graph holds
    the addresses of those workspaces: running one of the handles on a LARGER input afterwards re-allocates its
    workspace and invalidates the graph."""

    def __init__(self, net, x):
        self.net = net
        self.x = x.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            net.forward(self.x)             # sizes every workspace, on the stream family the capture will use
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.out = net.forward(self.x)

    def replay(self, x=None):
        if x is not None:
            self.x.copy_(x)
        self.graph.replay()
        return self.out


class _ShapeOnly:
    """Stands for the fp32 output of a chained layer that was not written: the next layer needs its shape only."""

    def __init__(self, shape, device):
        self.shape, self.device = tuple(shape), device


class ResNet20:
    def __init__(self, cfg, device="cuda"):
        self.bits = cfg["bits"]
        self.lut = B.Lut(cfg["lut"], self.bits)
        self.plan = resnet20_plan()
        self.qws = [quantize_weights(torch.from_numpy(w).to(device), self.bits) for w in cfg["convs"]]
        # the weights are static: combine them with the table once (Sec. III-B / III-C)
        self.pws = [B.adapt_weights_pack_conv2d(self.lut, qw) for qw, _ in self.qws]
        self.qfw, self.s_fw = quantize_weights(torch.from_numpy(cfg["fc_w"]).to(device), self.bits)
        self.p_fw = B.adapt_weights_pack_linear(self.lut, self.qfw)
        self.fc_b = torch.from_numpy(cfg["fc_b"]).to(device)
        self.scales = None
        self.macs = None
        self.chain = True           # frozen scales: every layer also writes the next layer's quantised input copy
        self._prepared = None       # input shape the chained buffers were prepared for
        self._needs_out = set()     # layers that need their fp32 output buffer even when nobody reads it

    def _prepare_chain(self, x):
        """Fix the place and layout of every convolution's input copy (all but the first receive it from the layer before)."""
        n, _, h, w = x.shape
        for i, (cin, cout, st) in enumerate(self.plan):
            if i > 0:
                B.adapt_conv2d_chain_prepare(self.pws[i], n, h, w, (st, st), (1, 1))
            h, w = (h + 2 - 3) // st + 1, (w + 2 - 3) // st + 1
        self._prepared = tuple(x.shape)

    def _conv(self, i, x, used, keep, relu=False, residual=None, want_out=True):
        """conv (+ ReLU).  Once the scales are frozen and nobody asks for the integer sums, the layer runs as one
        fused call (quantise while laying out the input, rescale + ReLU inside the product kernel)."""
        bits = self.bits
        st = self.plan[i][2]
        if self.scales is not None and keep is None:
            s_x = self.scales[i]
            used.append(s_x)
            if self.chain:
                # the input copy of every layer but the first is already in place (the layer before wrote it, quantised with
                # this layer's scale, from its epilogue); x is only needed for its shape
                n, _, h, w = x.shape
                ho, wo = (h + 2 - 3) // st + 1, (w + 2 - 3) // st + 1
                shape = (n, self.plan[i][1], ho, wo)
                last = i + 1 == len(self.plan)
                # a layer whose fp32 output nobody reads (only the next layer's copy is wanted) passes no output buffer,
                # unless its shape finishes the sums in a separate pass (found out on the first pass, remembered)
                skip = (not want_out) and (not last) and i not in self._needs_out
                for attempt in (0, 1):
                    out = None if skip else torch.empty(shape, dtype=torch.float32, device=x.device)
                    try:
                        B.adapt_conv2d_layer_chain_f32(self.pws[i], x if i == 0 else None, s_x, _f(s_x) * _f(self.qws[i][1]), out, (st, st),
                                                       (1, 1), act=B.ACT_RELU if relu else B.ACT_NONE, residual=residual,
                                                       next_pw=None if last else self.pws[i + 1],
                                                       s_next=1.0 if last else self.scales[i + 1], in_shape=(n, h, w))
                    except B.AdaptError as e:
                        if not (skip and e.code == -2):
                            raise
                        self._needs_out.add(i)
                        skip = False
                        continue
                    break
                return out if out is not None else _ShapeOnly(shape, x.device)
            return B.adapt_conv2d_layer_f32(self.pws[i], x, s_x, _f(s_x) * _f(self.qws[i][1]), (st, st), (1, 1),
                                            act=B.ACT_RELU if relu else B.ACT_NONE, residual=residual)
        s_x = calibrated_scale(x, bits) if self.scales is None else self.scales[i]
        used.append(s_x)
        qx = B.adapt_quantize_f32(x, s_x, bits)
        acc = B.adapt_approx_conv2d_packed(self.pws[i], qx, (st, st), (1, 1))
        if keep is not None:
            keep.append(acc)
        n, c, h, w = acc.shape
        y = B.adapt_dequant_i32(acc, _f(s_x) * _f(self.qws[i][1]), n, c, h * w)
        if residual is not None:
            return B.adapt_add_f32(y, residual, relu=relu)
        return B.adapt_relu_f32(y, out=y) if relu else y

    def forward(self, x, keep=None):
        used = []
        if self.scales is not None and keep is None and self.chain and self._prepared != tuple(x.shape):
            self._prepare_chain(x)
        x = self._conv(0, x, used, keep, relu=True)
        i = 1
        while i < len(self.plan):
            cin, cout, stride = self.plan[i]
            y = self._conv(i, x, used, keep, relu=True, want_out=False)     # (read only by the next layer, through its copy)
            sc = x if (stride == 1 and cin == cout) else B.adapt_shortcut_a_f32(x, cout)
            x = self._conv(i + 1, y, used, keep, relu=True, residual=sc)      # residual add + ReLU in the layer's epilogue
            i += 2
        pooled = B.adapt_avgpool_hw_f32(x)
        s_p = calibrated_scale(pooled, self.bits) if self.scales is None else self.scales[len(self.plan)]
        used.append(s_p)
        if self.scales is not None and keep is None:
            logits = B.adapt_linear_layer_f32(self.p_fw, pooled, s_p, _f(s_p) * _f(self.s_fw), self.fc_b)
            return dict(logits=logits, fc_acc=None, feat=x, scales=used)
        qp = B.adapt_quantize_f32(pooled, s_p, self.bits)
        acc = B.adapt_approx_linear_packed(self.p_fw, qp)
        logits = B.adapt_dequant_i32(acc, _f(s_p) * _f(self.s_fw), acc.shape[0], acc.shape[1], 1, self.fc_b)
        if self.scales is None:
            self.scales = used
        return dict(logits=logits, fc_acc=acc, feat=x, scales=used)


class LSTM:
    def __init__(self, cfg, device="cuda", fused_step=True):
        self.bits = cfg["bits"]
        self.lut = B.Lut(cfg["lut"], self.bits)
        self.q_wih, self.s_wih = quantize_weights(torch.from_numpy(cfg["w_ih"]).to(device), self.bits)
        self.q_whh, self.s_whh = quantize_weights(torch.from_numpy(cfg["w_hh"]).to(device), self.bits)
        self.p_wih = B.adapt_weights_pack_linear(self.lut, self.q_wih)      # one long product over all time steps
        self.p_whh = B.adapt_weights_pack_linear(self.lut, self.q_whh)      # 64-row products: pre-packed table-row offsets
        self.bias = torch.from_numpy(cfg["bias"]).to(device)
        self.Hs = cfg["w_hh"].shape[1]
        self.s_x = None
        self.fused_step = fused_step

    def forward(self, x):
        bits = self.bits
        T, Bn, I = x.shape
        Q = (1 << (bits - 1)) - 1
        if self.s_x is None:
            self.s_x = calibrated_scale(x, bits)          # over the whole [T, B, I] input
        s_h = _f(1.0) / _f(Q)
        qx = B.adapt_quantize_f32(x, self.s_x, bits).view(T * Bn, I)
        acc_ih = B.adapt_approx_linear_packed(self.p_wih, qx).view(T, Bn, 4 * self.Hs)
        hs = torch.empty((T, Bn, self.Hs), dtype=torch.float32, device=x.device)
        h = torch.zeros((Bn, self.Hs), dtype=torch.float32, device=x.device)
        c = torch.zeros((Bn, self.Hs), dtype=torch.float32, device=x.device)
        qh = torch.empty((Bn, self.Hs), dtype=torch.int8, device=x.device)
        acc_hh = torch.empty((Bn, 4 * self.Hs), dtype=torch.int32, device=x.device)
        s_ih = _f(self.s_x) * _f(self.s_wih)
        s_hh = _f(s_h) * _f(self.s_whh)
        B.adapt_quantize_f32(h, s_h, bits, out=qh)
        qh2 = torch.empty_like(qh)
        acc_last = None
        for t in range(T):
            h = hs[t]
            if self.fused_step:
                # product, cell and the next step's quantised h in one kernel; shapes it does not cover are refused
                # with UNSUPPORTED and take the two calls below
                try:
                    B.adapt_lstm_step_f32(self.p_whh, qh, acc_ih[t], s_ih, s_hh, s_h, self.bias, c, h, qh2)
                    qh, qh2 = qh2, qh
                    continue
                except B.AdaptError as e:
                    if e.code != -2:
                        raise
                    self.fused_step = False
            B.adapt_approx_linear_packed(self.p_whh, qh, out=acc_hh)
            acc_last = acc_hh
            # the cell also writes the quantised h that the next step multiplies
            B.adapt_lstm_cell_q_f32(acc_ih[t], acc_hh, s_ih, s_hh, self.bias, c, h, qh, s_h, bits)
        return dict(hs=hs, c=c, acc_ih=acc_ih, acc_hh_last=acc_last, s_x=self.s_x, s_h=s_h)


class Recurrent:
    """Single-layer GRU ("gru") or plain tanh recurrent layer ("rnn") (Sec. III-B "RNN Layer"): the input products of all
    time steps as one long table product, then per step the hidden-state product (pre-packed row offsets) and the cell
    kernel, which also writes the quantised h that the next step multiplies; where the shape allows the step is one
    fused kernel."""

    def __init__(self, cfg, kind, device="cuda", fused_step=True):
        self.kind = kind
        self.fused_step = fused_step
        self.gates = {"gru": 3, "rnn": 1}[kind]
        self.bits = cfg["bits"]
        self.lut = B.Lut(cfg["lut"], self.bits)
        self.q_wih, self.s_wih = quantize_weights(torch.from_numpy(cfg["w_ih"]).to(device), self.bits)
        self.q_whh, self.s_whh = quantize_weights(torch.from_numpy(cfg["w_hh"]).to(device), self.bits)
        self.p_wih = B.adapt_weights_pack_linear(self.lut, self.q_wih)
        self.p_whh = B.adapt_weights_pack_linear(self.lut, self.q_whh)
        if kind == "gru":
            self.b_ih = torch.from_numpy(cfg["b_ih"]).to(device)
            self.b_hh = torch.from_numpy(cfg["b_hh"]).to(device)
        else:
            self.bias = torch.from_numpy(cfg["bias"]).to(device)
        self.Hs = cfg["w_hh"].shape[1]
        self.s_x = None

    def forward(self, x):
        bits, G = self.bits, self.gates
        T, Bn, I = x.shape
        Q = (1 << (bits - 1)) - 1
        if self.s_x is None:
            self.s_x = calibrated_scale(x, bits)          # over the whole [T, B, I] input
        s_h = _f(1.0) / _f(Q)
        qx = B.adapt_quantize_f32(x, self.s_x, bits).view(T * Bn, I)
        acc_ih = B.adapt_approx_linear_packed(self.p_wih, qx).view(T, Bn, G * self.Hs)
        hs = torch.empty((T, Bn, self.Hs), dtype=torch.float32, device=x.device)
        h = torch.zeros((Bn, self.Hs), dtype=torch.float32, device=x.device)
        qh = torch.empty((Bn, self.Hs), dtype=torch.int8, device=x.device)
        acc_hh = torch.empty((Bn, G * self.Hs), dtype=torch.int32, device=x.device)
        s_ih = _f(self.s_x) * _f(self.s_wih)
        s_hh = _f(s_h) * _f(self.s_whh)
        B.adapt_quantize_f32(h, s_h, bits, out=qh)
        qh2 = torch.empty_like(qh)
        for t in range(T):
            if self.fused_step:
                # product, cell and the next step's quantised h in one kernel; shapes it does not cover are refused
                # with UNSUPPORTED and take the two calls below
                try:
                    if self.kind == "gru":
                        B.adapt_gru_step_f32(self.p_whh, qh, acc_ih[t], s_ih, s_hh, s_h, self.b_ih, self.b_hh, h, hs[t], qh2)
                    else:
                        B.adapt_rnn_step_f32(self.p_whh, qh, acc_ih[t], s_ih, s_hh, s_h, self.bias, hs[t], qh2)
                    qh, qh2 = qh2, qh
                    h = hs[t]
                    continue
                except B.AdaptError as e:
                    if e.code != -2:
                        raise
                    self.fused_step = False
            B.adapt_approx_linear_packed(self.p_whh, qh, out=acc_hh)
            if self.kind == "gru":
                B.adapt_gru_cell_f32(acc_ih[t], acc_hh, s_ih, s_hh, self.b_ih, self.b_hh, h, hs[t], qh, s_h, bits)
            else:
                B.adapt_rnn_cell_f32(acc_ih[t], acc_hh, s_ih, s_hh, self.bias, hs[t], False, qh, s_h, bits)
            h = hs[t]
        return dict(hs=hs, acc_ih=acc_ih, acc_hh_last=acc_hh, s_x=self.s_x, s_h=s_h)


class SeparableConv:
    """Separable convolution (Sec. III-B, eq. (1)): depthwise table-lookup convolution (groups = Cin), then the
    pointwise 1x1 convolution as a fused layer call."""

    def __init__(self, cfg, device="cuda"):
        self.bits = cfg["bits"]
        self.lut = B.Lut(cfg["lut"], self.bits)
        self.q_dw, self.s_dw = quantize_weights(torch.from_numpy(cfg["w_dw"]).to(device), self.bits)
        self.q_pw, self.s_pw = quantize_weights(torch.from_numpy(cfg["w_pw"]).to(device), self.bits)
        self.p_pw = B.adapt_weights_pack_conv2d(self.lut, self.q_pw)
        self.stride, self.pad = cfg["stride"], cfg["pad"]
        self.scales = None
        self._chain_shape = None

    def _forward_fused(self, x, keep_y):
        """Frozen scales: the depthwise layer quantises x itself and writes the pointwise layer's input copy
        (and y only when asked for), then the pointwise layer runs on that copy: two kernels in all."""
        s_x, s_y = self.scales
        n, cin, h, w = x.shape
        kh, kw = self.q_dw.shape[2:]
        ho, wo = B.conv_out_hw(h, w, kh, kw, self.stride, self.stride, self.pad, self.pad, 1, 1)
        shape = (n, ho, wo)
        if self._chain_shape != shape:
            B.adapt_conv2d_chain_prepare(self.p_pw, n, ho, wo)
            self._chain_shape = shape
        y = B.adapt_conv2d_grouped_layer_f32(self.lut, x, self.q_dw, s_x, _f(s_x) * _f(self.s_dw), (self.stride, self.stride),
                                             (self.pad, self.pad), groups=cin, want_out=keep_y, next_pw=self.p_pw, s_next=s_y)
        out = torch.empty((n, self.q_pw.shape[0], ho, wo), dtype=torch.float32, device=x.device)
        B.adapt_conv2d_layer_chain_f32(self.p_pw, None, s_y, _f(s_y) * _f(self.s_pw), out, in_shape=(n, ho, wo))
        return dict(out=out, y=y, scales=[s_x, s_y])

    def forward(self, x, fused=True, keep_y=False):
        bits = self.bits
        cin = x.shape[1]
        if fused and self.scales is not None:
            return self._forward_fused(x, keep_y)
        s_x = self.scales[0] if self.scales is not None else calibrated_scale(x, bits)
        qx = B.adapt_quantize_f32(x, s_x, bits)
        acc_dw = B.adapt_approx_conv2d(self.lut, qx, self.q_dw, (self.stride, self.stride), (self.pad, self.pad), groups=cin)
        n, c, h, w = acc_dw.shape
        y = B.adapt_dequant_i32(acc_dw, _f(s_x) * _f(self.s_dw), n, c, h * w)
        s_y = self.scales[1] if self.scales is not None else calibrated_scale(y, bits)
        out = B.adapt_conv2d_layer_f32(self.p_pw, y, s_y, _f(s_y) * _f(self.s_pw))
        if self.scales is None:
            self.scales = [s_x, s_y]
        return dict(out=out, y=y, acc_dw=acc_dw, scales=[s_x, s_y])


class DCGAN:
    def __init__(self, cfg, device="cuda", chain=True):
        self.chain = chain
        self._chain_shape = None
        self.bits = cfg["bits"]
        self.lut = B.Lut(cfg["lut"], self.bits)
        self.plan = cfg["plan"]
        self.qws = [quantize_weights(torch.from_numpy(w).to(device), self.bits) for w in cfg["ws"]]
        self.pws = [B.adapt_weights_pack_conv_transpose2d(self.lut, qw, s) for (qw, _), (_, _, s, _) in zip(self.qws, self.plan)]
        self.scales = None

    def _forward_chained(self, z):
        """Frozen scales: every layer writes the next layer's quantised input copy in its epilogue (one kernel per layer
        after the first).  Returns None when a layer's geometry cannot be prepared (the per-layer calls serve it then)."""
        n = z.shape[0]
        nl = len(self.plan)
        shapes = [tuple(z.shape)]
        for i, (cin, cout, s, p) in enumerate(self.plan):
            h, w = shapes[-1][2:]
            k = self.qws[i][0].shape[2]
            shapes.append((n, cout, (h - 1) * s - 2 * p + k, (w - 1) * s - 2 * p + k))
        if self._chain_shape != shapes[0]:
            try:
                for i in range(1, nl):
                    B.adapt_conv_transpose2d_chain_prepare(self.pws[i], n, shapes[i][2], shapes[i][3], self.plan[i][3])
            except B.AdaptError as e:
                if e.code != -2:
                    raise
                self.chain = False
                return None
            # only the last layer's fp32 output is read; the others get a buffer only if their shape needs one
            self._outs = [None] * (nl - 1) + [torch.empty(shapes[nl], dtype=torch.float32, device=z.device)]
            self._chain_shape = shapes[0]
        x = z
        for i, (cin, cout, s, p) in enumerate(self.plan):
            s_x = self.scales[i]
            nxt = self.pws[i + 1] if i + 1 < nl else None
            for attempt in (0, 1):
                try:
                    B.adapt_conv_transpose2d_layer_chain_f32(self.pws[i], x if i == 0 else None, s_x, _f(s_x) * _f(self.qws[i][1]),
                                                             self._outs[i], p, act=B.ACT_TANH if i == nl - 1 else B.ACT_RELU, next_pw=nxt,
                                                             s_next=self.scales[i + 1] if nxt is not None else 1.0,
                                                             in_shape=(n, shapes[i][2], shapes[i][3]))
                except B.AdaptError as e:
                    if not (self._outs[i] is None and e.code == -2):
                        raise
                    self._outs[i] = torch.empty(shapes[i + 1], dtype=torch.float32, device=z.device)
                    continue
                break
        return self._outs[-1]

    def forward(self, z, keep=None):
        used = []
        x = z
        nl = len(self.plan)
        acc = None
        if self.chain and self.scales is not None and keep is None:
            out = self._forward_chained(z)
            if out is not None:
                return dict(out=out, scales=list(self.scales), last_acc=None)
        for i, (cin, cout, s, p) in enumerate(self.plan):
            if self.scales is not None and keep is None:        # frozen scales: one fused call per layer
                s_x = self.scales[i]
                used.append(s_x)
                x = B.adapt_conv_transpose2d_layer_f32(self.pws[i], x, s_x, _f(s_x) * _f(self.qws[i][1]), p,
                                                       act=B.ACT_TANH if i == nl - 1 else B.ACT_RELU)
                continue
            s_x = calibrated_scale(x, self.bits) if self.scales is None else self.scales[i]
            used.append(s_x)
            qx = B.adapt_quantize_f32(x, s_x, self.bits)
            acc = B.adapt_approx_conv_transpose2d_packed(self.pws[i], qx, p)
            if keep is not None:
                keep.append(acc)
            n, c, h, w = acc.shape
            y = B.adapt_dequant_i32(acc, _f(s_x) * _f(self.qws[i][1]), n, c, h * w)
            x = B.adapt_tanh_f32(y, out=y) if i == nl - 1 else B.adapt_relu_f32(y, out=y)
        if self.scales is None:
            self.scales = used
        return dict(out=x, scales=used, last_acc=acc)


def lut_macs_resnet20(batch: int) -> int:
    macs, hw = 0, 32
    for cin, cout, s in resnet20_plan():
        hw = hw // s
        macs += cout * hw * hw * cin * 9
    return batch * (macs + 64 * 10)


def lut_macs_lstm(T, Bn, I, Hs) -> int:
    return T * Bn * (I + Hs) * 4 * Hs


def lut_macs_dcgan(batch: int, plan) -> int:
    macs, hw = 0, 1
    for i, (cin, cout, s, p) in enumerate(plan):
        macs += hw * hw * cin * cout * 16
        hw = (hw - 1) * s - 2 * p + 4
    return batch * macs
