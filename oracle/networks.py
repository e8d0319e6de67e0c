"""Oracle runners for the network-shaped workloads (CNN, LSTM, GAN families of
Sec. V, Table I), built only from the layer definitions in `oracle.c`.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Every approximate layer is  quantise -> table-lookup matrix product ->
dequantise  (Sec. III-A, IV).  Activation scales come from max-abs calibration
(the simple scale choice named in Sec. III-A) taken *progressively through the
approximate pipeline* on the calibration batch; weights use one max-abs scale
per tensor.  All scale arithmetic is fp32.
"""
from __future__ import annotations

import numpy as np

import oracle as orc


def _f(x):
    return np.float32(x)


def quantize_weights(w, bits):
    s = orc.scale_from_amax(orc.absmax(w), bits)
    return orc.quantize(w, s, bits), s


def conv_layer(lut, bits, x, qw, s_w, stride, pad, s_x=None, threads=1):
    """fp32 in -> fp32 out through one approximate 3x3/any conv; returns (y, s_x, q_x, acc)."""
    if s_x is None:
        s_x = orc.scale_from_amax(orc.absmax(x), bits)
    qx = orc.quantize(x, s_x, bits)
    acc = orc.approx_conv2d(lut, bits, qx, qw, (stride, stride), (pad, pad), threads=threads)
    n, c, h, w = acc.shape
    y = orc.dequant(acc, _f(s_x) * _f(s_w), n, c, h * w)
    return y, s_x, qx, acc


def resnet20(cfg, scales=None, threads=1, keep=False):
    """ResNet-20-style CNN without normalisation layers: conv-ReLU stem, nine
    two-conv residual blocks (parameter-free shortcut when the shape changes),
    global average pool, approximate linear classifier with bias."""
    from paper_2203_04071_amd.workloads import resnet20_plan
    bits, lut = cfg["bits"], cfg["lut"]
    plan = resnet20_plan()
    qws = [quantize_weights(w, bits) for w in cfg["convs"]]
    used = []
    trace = []

    def layer(i, x):
        s_in = None if scales is None else scales[i]
        y, s_x, qx, acc = conv_layer(lut, bits, x, qws[i][0], qws[i][1], plan[i][2], 1, s_in, threads)
        used.append(s_x)
        if keep:
            trace.append(acc)
        return y

    x = orc.relu(layer(0, cfg["x"]))
    i = 1
    while i < len(plan):
        cin, cout, stride = plan[i]
        y = orc.relu(layer(i, x))
        z = layer(i + 1, y)
        sc = x if (stride == 1 and cin == cout) else orc.shortcut_a(x, cout)
        x = orc.relu(orc.add(z, sc))
        i += 2
    pooled = orc.avgpool_hw(x)
    qfw, s_fw = quantize_weights(cfg["fc_w"], bits)
    s_p = orc.scale_from_amax(orc.absmax(pooled), bits) if scales is None else scales[len(plan)]
    used.append(s_p)
    qp = orc.quantize(pooled, s_p, bits)
    acc = orc.approx_linear(lut, bits, qp, qfw, threads)
    logits = orc.dequant(acc, _f(s_p) * _f(s_fw), acc.shape[0], acc.shape[1], 1, cfg["fc_b"])
    return dict(logits=logits, fc_acc=acc, scales=used, feat=x, trace=trace)


def lstm(cfg, threads=1, steps=None):
    """Single-layer LSTM whose gate pre-activations are approximate linear layers
    (Sec. III-B "RNN Layer"); sigmoid/tanh and the cell update in fp32."""
    bits, lut = cfg["bits"], cfg["lut"]
    x = cfg["x"]
    T, B, I = x.shape
    if steps is not None:
        T = min(T, steps)
    Hs = cfg["w_hh"].shape[1]
    Q = (1 << (bits - 1)) - 1
    q_wih, s_wih = quantize_weights(cfg["w_ih"], bits)
    q_whh, s_whh = quantize_weights(cfg["w_hh"], bits)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)       # over the whole [T, B, I] input
    s_h = _f(1.0) / _f(Q)                                # |h| < 1
    qx = orc.quantize(x[:T], s_x, bits).reshape(T * B, I)
    acc_ih = orc.approx_linear(lut, bits, qx, q_wih, threads).reshape(T, B, 4 * Hs)
    h = np.zeros((B, Hs), dtype=np.float32)
    c = np.zeros((B, Hs), dtype=np.float32)
    hs = np.empty((T, B, Hs), dtype=np.float32)
    acc_hh_last = None
    for t in range(T):
        qh = orc.quantize(h, s_h, bits)
        acc_hh = orc.approx_linear(lut, bits, qh, q_whh, threads)
        h, c = orc.lstm_cell(acc_ih[t], acc_hh, _f(s_x) * _f(s_wih), _f(s_h) * _f(s_whh), cfg["bias"], c)
        hs[t] = h
        acc_hh_last = acc_hh
    return dict(hs=hs, c=c, acc_ih=acc_ih, acc_hh_last=acc_hh_last, s_x=s_x, s_h=s_h, s_wih=s_wih, s_whh=s_whh)


def dcgan(cfg, scales=None, threads=1, keep=False):
    """DCGAN-style generator: five approximate transposed convolutions, ReLU
    between them, tanh at the end; no normalisation layers."""
    bits, lut = cfg["bits"], cfg["lut"]
    x = cfg["z"]
    used, accs = [], []
    nl = len(cfg["plan"])
    for i, ((cin, cout, s, p), w) in enumerate(zip(cfg["plan"], cfg["ws"])):
        qw, s_w = quantize_weights(w, bits)
        s_x = orc.scale_from_amax(orc.absmax(x), bits) if scales is None else scales[i]
        used.append(s_x)
        qx = orc.quantize(x, s_x, bits)
        acc = orc.approx_conv_transpose2d(lut, bits, qx, qw, s, p, threads)
        if keep:
            accs.append(acc)
        n, c, h, wd = acc.shape
        y = orc.dequant(acc, _f(s_x) * _f(s_w), n, c, h * wd)
        x = orc.tanh(y) if i == nl - 1 else orc.relu(y)
    return dict(out=x, scales=used, accs=accs, last_acc=acc)


def _recurrent_inputs(cfg, gates, threads, steps):
    """Shared front part of the recurrent runners: quantised weights, scales, and the input sums of all steps."""
    bits, lut = cfg["bits"], cfg["lut"]
    x = cfg["x"]
    T, B, I = x.shape
    if steps is not None:
        T = min(T, steps)
    Hs = cfg["w_hh"].shape[1]
    assert cfg["w_ih"].shape == (gates * Hs, I) and cfg["w_hh"].shape == (gates * Hs, Hs)
    Q = (1 << (bits - 1)) - 1
    q_wih, s_wih = quantize_weights(cfg["w_ih"], bits)
    q_whh, s_whh = quantize_weights(cfg["w_hh"], bits)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)       # over the whole [T, B, I] input
    s_h = _f(1.0) / _f(Q)                                # |h| < 1
    qx = orc.quantize(x[:T], s_x, bits).reshape(T * B, I)
    acc_ih = orc.approx_linear(lut, bits, qx, q_wih, threads).reshape(T, B, gates * Hs)
    return T, B, Hs, q_whh, s_wih, s_whh, s_x, s_h, acc_ih


def gru(cfg, threads=1, steps=None):
    """Single-layer GRU whose gate pre-activations are approximate linear layers (Sec. III-B "RNN Layer");
    gates and the state update in fp32.  cfg: x [T][B][I], w_ih [3 Hs][I], w_hh [3 Hs][Hs], b_ih, b_hh [3 Hs]."""
    bits, lut = cfg["bits"], cfg["lut"]
    T, B, Hs, q_whh, s_wih, s_whh, s_x, s_h, acc_ih = _recurrent_inputs(cfg, 3, threads, steps)
    h = np.zeros((B, Hs), dtype=np.float32)
    hs = np.empty((T, B, Hs), dtype=np.float32)
    acc_hh = None
    for t in range(T):
        qh = orc.quantize(h, s_h, bits)
        acc_hh = orc.approx_linear(lut, bits, qh, q_whh, threads)
        h = orc.gru_cell(acc_ih[t], acc_hh, _f(s_x) * _f(s_wih), _f(s_h) * _f(s_whh), cfg["b_ih"], cfg["b_hh"], h)
        hs[t] = h
    return dict(hs=hs, acc_ih=acc_ih, acc_hh_last=acc_hh, s_x=s_x, s_h=s_h, s_wih=s_wih, s_whh=s_whh)


def rnn(cfg, threads=1, steps=None):
    """Single-layer tanh recurrent layer, h_t = tanh(W_ih x_t + W_hh h_(t-1) + b) with approximate linear layers
    (Sec. III-B "RNN Layer").  cfg: x [T][B][I], w_ih [Hs][I], w_hh [Hs][Hs], bias [Hs]."""
    bits, lut = cfg["bits"], cfg["lut"]
    T, B, Hs, q_whh, s_wih, s_whh, s_x, s_h, acc_ih = _recurrent_inputs(cfg, 1, threads, steps)
    h = np.zeros((B, Hs), dtype=np.float32)
    hs = np.empty((T, B, Hs), dtype=np.float32)
    acc_hh = None
    for t in range(T):
        qh = orc.quantize(h, s_h, bits)
        acc_hh = orc.approx_linear(lut, bits, qh, q_whh, threads)
        h = orc.rnn_cell(acc_ih[t], acc_hh, _f(s_x) * _f(s_wih), _f(s_h) * _f(s_whh), cfg["bias"], relu=False)
        hs[t] = h
    return dict(hs=hs, acc_ih=acc_ih, acc_hh_last=acc_hh, s_x=s_x, s_h=s_h, s_wih=s_wih, s_whh=s_whh)


def separable_conv(cfg, scales=None, threads=1):
    """Separable convolution (Sec. III-B "Separable convolution", eq. (1)): a depthwise convolution (groups = Cin)
    followed by a pointwise 1x1 convolution, each an approximate layer of its own (quantise -> table-lookup
    convolution -> dequantise).  cfg: x [N][Cin][H][W], w_dw [Cin][1][kh][kw], w_pw [Cout][Cin][1][1], stride, pad."""
    bits, lut = cfg["bits"], cfg["lut"]
    x = cfg["x"]
    Cin = x.shape[1]
    q_dw, s_dw = quantize_weights(cfg["w_dw"], bits)
    q_pw, s_pw = quantize_weights(cfg["w_pw"], bits)
    s_x = scales[0] if scales is not None else orc.scale_from_amax(orc.absmax(x), bits)
    qx = orc.quantize(x, s_x, bits)
    st, pd = cfg["stride"], cfg["pad"]
    acc_dw = orc.approx_conv2d(lut, bits, qx, q_dw, (st, st), (pd, pd), groups=Cin, threads=threads)
    n, c, h, w = acc_dw.shape
    y = orc.dequant(acc_dw, _f(s_x) * _f(s_dw), n, c, h * w)
    s_y = scales[1] if scales is not None else orc.scale_from_amax(orc.absmax(y), bits)
    qy = orc.quantize(y, s_y, bits)
    acc_pw = orc.approx_conv2d(lut, bits, qy, q_pw, threads=threads)
    n, c, h, w = acc_pw.shape
    out = orc.dequant(acc_pw, _f(s_y) * _f(s_pw), n, c, h * w)
    return dict(out=out, y=y, acc_dw=acc_dw, acc_pw=acc_pw, scales=[s_x, s_y], s_dw=s_dw, s_pw=s_pw)
