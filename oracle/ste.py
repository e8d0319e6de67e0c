"""CPU oracle: backward pass of an approximate linear layer under the straight-through estimator.

TEST INFRASTRUCTURE ONLY (see the package header): nothing of the product path imports this file.

What is computed (Sec. III-A, "Retraining": training continues through fake-quantisation modules, with the
straight-through estimator as the derivative of the quantiser; the forward pass goes through the multiplier table).
The estimator replaces two derivatives by that of the identity:

* the quantiser x -> s * clamp(rint(x / s), -Q, Q) passes a gradient unchanged where its clamp did not act,
  |rint(x / s)| <= Q, and passes nothing where it did;
* the table T[a][w] is differentiated as the exact product a * w that it approximates.

For y[m][n] = sum_k x^[m][k] * w^[n][k] + b[n], with x^ = s_x * q(x) and w^ = s_w * q(w) the fake-quantised operands,
that gives

    dx[m][k] = inside(x[m][k], s_x) * sum_n dy[m][n] * w^[n][k]
    dw[n][k] = inside(w[n][k], s_w) * sum_m dy[m][n] * x^[m][k]
    db[n]    = sum_m dy[m][n]

The quantiser's decisions (code, inside / clipped) are taken in fp32 exactly as the forward quantiser takes them
(IEEE division, round half to even); a fake-quantised value is one fp32 product code * s; the three sums are formed in
fp64.  Readings where the paper is silent: "inside" is decided on the rounded code, so the element that defines a
max-abs scale always keeps its gradient; NaN inputs get no gradient.
"""
from __future__ import annotations

import numpy as np


def _codes_f32(x, scale):
    """rint(x / s) in fp32, before the clamp."""
    x = np.asarray(x, dtype=np.float32)
    s = np.float32(scale)
    with np.errstate(invalid="ignore", over="ignore"):
        return np.rint(x / s).astype(np.float32)


def clip_inside(x, scale, bits) -> np.ndarray:
    """True where the quantiser's clamp did not act on x."""
    Q = np.float32((1 << (int(bits) - 1)) - 1)
    r = _codes_f32(x, scale)
    with np.errstate(invalid="ignore"):
        return np.abs(r) <= Q              # False for NaN


def fake_quant(x, scale, bits) -> np.ndarray:
    """s * clamp(rint(x / s), -Q, Q) as fp32 (NaN -> 0, like the forward quantiser)."""
    Q = np.float32((1 << (int(bits) - 1)) - 1)
    r = _codes_f32(x, scale)
    r = np.where(np.isnan(r), np.float32(0), r)
    r = np.minimum(np.maximum(r, -Q), Q).astype(np.float32)
    return (r * np.float32(scale)).astype(np.float32)


def ste_linear_backward(dy, x, w, s_x, s_w, bits):
    """dy [M][N], x [M][K], w [N][K] (fp32) -> dx [M][K], dw [N][K], db [N] in fp64."""
    dy = np.asarray(dy, dtype=np.float32)
    x = np.asarray(x, dtype=np.float32)
    w = np.asarray(w, dtype=np.float32)
    M, N = dy.shape
    assert x.shape[0] == M and w.shape[0] == N and x.shape[1] == w.shape[1]
    dy64 = dy.astype(np.float64)
    xh = fake_quant(x, s_x, bits).astype(np.float64)
    wh = fake_quant(w, s_w, bits).astype(np.float64)
    dx = (dy64 @ wh) * clip_inside(x, s_x, bits)
    dw = (dy64.T @ xh) * clip_inside(w, s_w, bits)
    db = dy64.sum(axis=0)
    return dx, dw, db


def ste_linear_backward_bound(dy, x, w, s_x, s_w, bits):
    """sum of |terms| of each output: what an fp32 accumulation error is measured against."""
    dy64 = np.abs(np.asarray(dy, dtype=np.float32).astype(np.float64))
    xh = np.abs(fake_quant(x, s_x, bits).astype(np.float64))
    wh = np.abs(fake_quant(w, s_w, bits).astype(np.float64))
    return dy64 @ wh, dy64.T @ xh, dy64.sum(axis=0)


def sgd_step(w, g, lr) -> np.ndarray:
    """One plain SGD step in fp32 (Sec. V-A, "Quantization and retraining": the paper retrains with SGD): w - lr * g, the product rounded, then the difference."""
    w = np.asarray(w, dtype=np.float32)
    g = np.asarray(g, dtype=np.float32)
    prod = (np.float32(lr) * g).astype(np.float32)
    return (w - prod).astype(np.float32)


def _conv_out(H, k, s, p, d):
    return (H + 2 * p - d * (k - 1) - 1) // s + 1


def ste_conv2d_backward(dy, x, w, stride, pad, dil, s_x, s_w, bits, absolute=False):
    """Straight-through backward pass of an approximate 2-D convolution (groups = 1), tap by tap from the definition
    y[n][o][oy][ox] = sum_{c,ky,kx} x^[n][c][oy s - p + ky d][ox s - p + kx d] * w^[o][c][ky][kx] (zero outside the image):

        dw[o][c][ky][kx] = inside(w) * sum_{n,oy,ox} dy[n][o][oy][ox] * x^[n][c][oy s - p + ky d][ox s - p + kx d]
        dx[n][c][iy][ix] = inside(x) * sum over the (o, ky, kx, oy, ox) whose tap lands on (iy, ix) of dy * w^
        db[o]            = sum_{n,oy,ox} dy[n][o][oy][ox]

    dy [N][O][Ho][Wo], x [N][C][H][W], w [O][C][kh][kw] fp32 -> fp64 results.  absolute=True: the same sums over
    absolute values without the masks (what an fp32 accumulation error is measured against)."""
    dy = np.asarray(dy, dtype=np.float32).astype(np.float64)
    x32 = np.asarray(x, dtype=np.float32)
    w32 = np.asarray(w, dtype=np.float32)
    N, C, H, W = x32.shape
    O, C2, kh, kw = w32.shape
    (sh, sw), (ph, pw), (dh, dw_) = stride, pad, dil
    Ho, Wo = _conv_out(H, kh, sh, ph, dh), _conv_out(W, kw, sw, pw, dw_)
    assert C2 == C and dy.shape == (N, O, Ho, Wo)
    xh = fake_quant(x32, s_x, bits).astype(np.float64)
    wh = fake_quant(w32, s_w, bits).astype(np.float64)
    if absolute:
        dy, xh, wh = np.abs(dy), np.abs(xh), np.abs(wh)
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw))
    xp[:, :, ph:ph + H, pw:pw + W] = xh
    dxp = np.zeros_like(xp)
    dwt = np.zeros((O, C, kh, kw))
    for ky in range(kh):
        for kx in range(kw):
            ys = slice(ky * dh, ky * dh + (Ho - 1) * sh + 1, sh)
            xs = slice(kx * dw_, kx * dw_ + (Wo - 1) * sw + 1, sw)
            dwt[:, :, ky, kx] = np.einsum("nohw,nchw->oc", dy, xp[:, :, ys, xs])
            dxp[:, :, ys, xs] += np.einsum("nohw,oc->nchw", dy, wh[:, :, ky, kx])
    dx = dxp[:, :, ph:ph + H, pw:pw + W]
    db = dy.sum(axis=(0, 2, 3))
    if not absolute:
        dx = dx * clip_inside(x32, s_x, bits)
        dwt = dwt * clip_inside(w32, s_w, bits)
    return dx, dwt, db


def relu_backward(dy, y) -> np.ndarray:
    """Gradient through y = max(v, 0), the activation the approximate layers fuse: dy where y > 0, else 0 (fp32, exact)."""
    dy = np.asarray(dy, dtype=np.float32)
    y = np.asarray(y, dtype=np.float32)
    return np.where(y > 0, dy, np.float32(0)).astype(np.float32)
