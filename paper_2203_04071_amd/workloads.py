"""Seeded synthetic inputs for the approximate-multiplier hot path.

This module only *draws inputs* (tensors, weights, multiplier tables) from
numpy's counter-free `default_rng(seed)` streams.  It holds none of the
method's arithmetic (no quantiser, no table lookup, no dequantiser) and
imports neither the CPU oracle nor the HIP binding, so that both sides of
a parity test are fed byte-identical arrays.

The paper evaluates on CIFAR-10 / ImageNet / IMDB / MNIST / Fashion-MNIST
with trained models and EvoApprox multiplier tables (Sec. V, Tables I-III).
None of those is available offline; the generators below stand in for them
with the same layer families (CNN, LSTM, GAN), 8-bit default precision and
batch 128 for the CNN, and with the distributions the benchmark
configurations state.
"""
from __future__ import annotations

import numpy as np

DATA_SEED_BASE = 1234   # + config number
LUT_SEED_BASE = 4321    # + bits

# error amplitude of the synthetic approximate multiplier per bitwidth
LUT_ERR = {8: 64, 7: 32, 6: 8}


def make_lut(bits: int, err: int | None = None, seed: int | None = None,
             symmetric: bool = True) -> np.ndarray:
    """Synthetic approximate-multiplier table.

    Returns int32 [2^b, 2^b]; entry for signed operands (a, w), both in
    [-H, H-1] with H = 2^(b-1), sits at [a + H, w + H] and equals the exact
    product plus an integer error drawn uniformly from [-err, err].  With
    `symmetric` the error is drawn for a <= w and mirrored, so the table
    models a commutative multiplier.  Every entry gets an error, including
    the rows and columns of a zero operand.
    """
    if err is None:
        err = LUT_ERR.get(bits, max(1, (1 << (2 * bits - 2)) // 256))
    if seed is None:
        seed = LUT_SEED_BASE + bits
    n = 1 << bits
    h = n >> 1
    rng = np.random.default_rng(seed)
    e = rng.integers(-err, err + 1, size=(n, n), dtype=np.int64)
    if symmetric:
        e = np.triu(e) + np.triu(e, 1).T
    v = np.arange(-h, h, dtype=np.int64)
    t = v[:, None] * v[None, :] + e
    return np.ascontiguousarray(t.astype(np.int32))


def exact_lut(bits: int) -> np.ndarray:
    """Table of the exact multiplier (an input used by invariants, not a result)."""
    return make_lut(bits, err=0, seed=0)


def config1(seed: int = DATA_SEED_BASE + 1) -> dict:
    """Single approximate linear layer, uniform int8 operands (worst-case index spread)."""
    rng = np.random.default_rng(seed)
    a = rng.integers(-128, 128, size=(64, 256), dtype=np.int64).astype(np.int8)
    w = rng.integers(-128, 128, size=(128, 256), dtype=np.int64).astype(np.int8)
    return dict(bits=8, A=a, W=w, lut=make_lut(8), scale=np.float32(0.01), M=64, K=256, N=128)


def config2(seed: int = DATA_SEED_BASE + 2, batch: int = 32, cin: int = 64, cout: int = 64,
            hw: int = 32) -> dict:
    """3x3 stride-1 pad-1 convolution on Gaussian fp32 inputs, He-normal weights."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, cin, hw, hw), dtype=np.float32)
    std = np.float32(np.sqrt(2.0 / (cin * 9)))
    w = rng.standard_normal((cout, cin, 3, 3), dtype=np.float32) * std
    return dict(bits=8, x=x, w=w.astype(np.float32), lut=make_lut(8), stride=1, pad=1)


def resnet20_plan() -> list:
    """(cin, cout, stride) of the 19 3x3 convolutions of a CIFAR-style ResNet-20."""
    plan = [(3, 16, 1)]
    cin = 16
    for stage, cout in enumerate((16, 32, 64)):
        for block in range(3):
            s = 2 if (stage > 0 and block == 0) else 1
            plan.append((cin, cout, s))
            plan.append((cout, cout, 1))
            cin = cout
    return plan


def config3(seed: int = DATA_SEED_BASE + 3, batch: int = 128) -> dict:
    """ResNet-20-style CNN, random He-normal weights, N(0,1) 3x32x32 inputs."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, 3, 32, 32), dtype=np.float32)
    convs = []
    for cin, cout, s in resnet20_plan():
        std = np.float32(np.sqrt(2.0 / (cin * 9)))
        convs.append((rng.standard_normal((cout, cin, 3, 3), dtype=np.float32) * std).astype(np.float32))
    fc_w = (rng.standard_normal((10, 64), dtype=np.float32) * np.float32(np.sqrt(2.0 / 64))).astype(np.float32)
    fc_b = np.zeros(10, dtype=np.float32)
    return dict(bits=8, x=x, convs=convs, fc_w=fc_w, fc_b=fc_b, lut=make_lut(8))


def config4(seed: int = DATA_SEED_BASE + 4, seq: int = 100, batch: int = 64, isz: int = 512,
            hsz: int = 512) -> dict:
    """Single-layer LSTM; weights N(0, std 0.1); inputs N(0,1); 7-bit multiplier."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((seq, batch, isz), dtype=np.float32)
    w_ih = (rng.standard_normal((4 * hsz, isz), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    w_hh = (rng.standard_normal((4 * hsz, hsz), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    bias = np.zeros(4 * hsz, dtype=np.float32)
    return dict(bits=7, x=x, w_ih=w_ih, w_hh=w_hh, bias=bias, lut=make_lut(7))


DCGAN_PLAN = [  # (cin, cout, stride, pad) of the 4x4 transposed convolutions
    (100, 512, 1, 0),
    (512, 256, 2, 1),
    (256, 128, 2, 1),
    (128, 64, 2, 1),
    (64, 3, 2, 1),
]


def config5(bits: int = 8, seed: int = DATA_SEED_BASE + 5, batch: int = 256) -> dict:
    """DCGAN-style generator; weights N(0, 0.02); z ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((batch, 100, 1, 1), dtype=np.float32)
    ws = []
    for cin, cout, s, p in DCGAN_PLAN:
        ws.append((rng.standard_normal((cin, cout, 4, 4), dtype=np.float32) * np.float32(0.02)).astype(np.float32))
    return dict(bits=bits, z=z, ws=ws, lut=make_lut(bits), plan=list(DCGAN_PLAN))


def recurrent_workload(kind: str = "gru", seed: int = DATA_SEED_BASE + 40, seq: int = 20, batch: int = 16, isz: int = 128,
                       hsz: int = 128, bits: int = 8) -> dict:
    """Single-layer GRU ("gru": 3 gates, two bias vectors) or plain tanh recurrent layer ("rnn": one gate, one bias);
    weights N(0, std 0.1), biases N(0, std 0.05), inputs N(0, 1) — the recipe of the LSTM configuration."""
    gates = {"gru": 3, "rnn": 1}[kind]
    rng = np.random.default_rng(seed + (0 if kind == "gru" else 1))
    x = rng.standard_normal((seq, batch, isz), dtype=np.float32)
    w_ih = (rng.standard_normal((gates * hsz, isz), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    w_hh = (rng.standard_normal((gates * hsz, hsz), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    cfg = dict(bits=bits, x=x, w_ih=w_ih, w_hh=w_hh, lut=make_lut(bits))
    if kind == "gru":
        cfg["b_ih"] = (rng.standard_normal(3 * hsz, dtype=np.float32) * np.float32(0.05)).astype(np.float32)
        cfg["b_hh"] = (rng.standard_normal(3 * hsz, dtype=np.float32) * np.float32(0.05)).astype(np.float32)
    else:
        cfg["bias"] = (rng.standard_normal(hsz, dtype=np.float32) * np.float32(0.05)).astype(np.float32)
    return cfg


def separable_workload(seed: int = DATA_SEED_BASE + 42, batch: int = 8, cin: int = 32, cout: int = 64, hw: int = 16,
                       k: int = 3, stride: int = 1, bits: int = 8) -> dict:
    """Separable convolution block: depthwise k x k (groups = cin, pad k // 2) then pointwise 1 x 1; He-normal weights,
    inputs N(0, 1)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, cin, hw, hw), dtype=np.float32)
    w_dw = (rng.standard_normal((cin, 1, k, k), dtype=np.float32) * np.float32(np.sqrt(2.0 / (k * k)))).astype(np.float32)
    w_pw = (rng.standard_normal((cout, cin, 1, 1), dtype=np.float32) * np.float32(np.sqrt(2.0 / cin))).astype(np.float32)
    return dict(bits=bits, x=x, w_dw=w_dw, w_pw=w_pw, stride=stride, pad=k // 2, lut=make_lut(bits))


def lut_macs_conv2d(n, cin, h, w, cout, kh, kw, sh, sw, ph, pw, dh=1, dw=1, groups=1) -> int:
    """Number of table terms of a convolution, padded taps included."""
    ho = (h + 2 * ph - dh * (kh - 1) - 1) // sh + 1
    wo = (w + 2 * pw - dw * (kw - 1) - 1) // sw + 1
    return n * cout * ho * wo * (cin // groups) * kh * kw


def random_i8(rng, shape, bits=8, dist="uniform") -> np.ndarray:
    """int8 operands in the b-bit signed range, uniform or Gaussian-shaped."""
    h = 1 << (bits - 1)
    if dist == "uniform":
        v = rng.integers(-h, h, size=shape, dtype=np.int64)
    else:
        v = np.clip(np.rint(rng.standard_normal(shape) * (h / 5.2)), -h, h - 1).astype(np.int64)
    return v.astype(np.int8)
