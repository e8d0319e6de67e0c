"""Pins of the oracle's straight-through backward pass (Sec. III-A, "Retraining") against things other than itself:
an automatic-differentiation library, closed forms, and the quantiser's own special cases.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from oracle import ste


def _autograd_reference(dy, x, w, s_x, s_w, bits):
    """The same estimator written for torch.autograd in fp64: rounding is made transparent with the detach trick, the
    clamp keeps its own derivative (1 where it does not act, 0 where it does)."""
    Q = float((1 << (bits - 1)) - 1)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    bt = torch.zeros(w.shape[0], dtype=torch.float64, requires_grad=True)

    def fq(t, s):
        r = t / s
        r = r + (torch.round(r) - r).detach()
        return torch.clamp(r, -Q, Q) * s

    y = fq(xt, s_x) @ fq(wt, s_w).T + bt
    (y * torch.tensor(dy, dtype=torch.float64)).sum().backward()
    return xt.grad.numpy(), wt.grad.numpy(), bt.grad.numpy()


@pytest.mark.parametrize("bits,M,K,N,seed", [(8, 5, 7, 3, 0), (4, 9, 6, 11, 1), (12, 4, 33, 2, 2), (6, 1, 1, 1, 3)])
def test_backward_equals_autograd_of_fake_quantised_layer(bits, M, K, N, seed):
    rng = np.random.default_rng(seed)
    Q = (1 << (bits - 1)) - 1
    s_x, s_w = 2.0 ** -4, 2.0 ** -6           # powers of two: fp32 and fp64 take identical quantiser decisions
    # values on a grid of quarter steps: exact ties and values beyond the clipping range both occur
    def grid(shape, s):
        v = rng.integers(-4 * Q - 12, 4 * Q + 13, size=shape)
        edge = rng.random(shape) < 0.3                                      # a third of them around the clipping point
        v = np.where(edge, rng.choice([-1, 1], size=shape) * (4 * Q + rng.integers(-6, 7, size=shape)), v)
        return (v * 0.25 * s).astype(np.float32)

    x, w = grid((M, K), s_x), grid((N, K), s_w)
    dy = rng.standard_normal((M, N)).astype(np.float32)
    dx, dw, db = ste.ste_linear_backward(dy, x, w, s_x, s_w, bits)
    rx, rw, rb = _autograd_reference(dy, x, w, s_x, s_w, bits)
    assert (np.abs(x) > Q * s_x).any() or M * K < 4
    np.testing.assert_allclose(dx, rx, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dw, rw, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(db, rb, rtol=1e-12, atol=1e-14)


def test_one_hot_gradient_picks_rows_of_the_fake_quantised_operands():
    # dy = e(m0, n0): dx[m0] = w^[n0] where x is inside, dw[n0] = x^[m0] where w is inside, everything else 0.
    # w^ / x^ come from the C quantiser (pinned elsewhere), not from the routine under test.
    rng = np.random.default_rng(5)
    bits, M, K, N = 8, 6, 10, 4
    x = rng.standard_normal((M, K)).astype(np.float32) * 2
    w = rng.standard_normal((N, K)).astype(np.float32)
    s_x, s_w = np.float32(0.013), np.float32(0.0071)        # |x| reaches beyond 127 * 0.013 = 1.65
    m0, n0 = 4, 2
    dy = np.zeros((M, N), dtype=np.float32)
    dy[m0, n0] = 1.0
    dx, dw, db = ste.ste_linear_backward(dy, x, w, s_x, s_w, bits)
    xh = oracle.quantize(x, s_x, bits).astype(np.float32) * s_x
    wh = oracle.quantize(w, s_w, bits).astype(np.float32) * s_w
    in_x = np.abs(np.rint(x / s_x)) <= 127
    in_w = np.abs(np.rint(w / s_w)) <= 127
    assert not in_x.all()
    exp_dx = np.zeros((M, K)); exp_dx[m0] = wh[n0] * in_x[m0]
    exp_dw = np.zeros((N, K)); exp_dw[n0] = xh[m0] * in_w[n0]
    np.testing.assert_array_equal(dx, exp_dx)
    np.testing.assert_array_equal(dw, exp_dw)
    np.testing.assert_array_equal(db, np.eye(N)[n0])


def test_clip_decision_special_cases():
    x = np.array([127.5, 127.49, -127.5, 126.5, 1000.0, -127.0, np.nan, 0.0], dtype=np.float32)
    np.testing.assert_array_equal(ste.clip_inside(x, 1.0, 8), [False, True, False, True, False, True, False, True])
    # half to even: 7.5 -> 8 is clipped at 4 bits (Q = 7), 6.5 -> 6 is not
    np.testing.assert_array_equal(ste.clip_inside(np.array([7.5, 6.5, -7.5, 7.4], dtype=np.float32), 1.0, 4), [False, True, False, True])
    np.testing.assert_array_equal(ste.fake_quant(x, 1.0, 8), [127, 127, -127, 126, 127, -127, 0, 0])


@pytest.mark.parametrize("bits", [4, 7, 8, 12])
def test_element_that_sets_a_max_abs_scale_keeps_its_gradient(bits):
    for seed in range(50):
        x = np.random.default_rng(seed).standard_normal(257).astype(np.float32) * np.float32(1 + seed)
        s = oracle.scale_from_amax(oracle.absmax(x), bits)
        inside = ste.clip_inside(x, s, bits)
        assert inside.all()
        np.testing.assert_array_equal(ste.fake_quant(x, s, bits), oracle.quantize_i16(x, s, bits).astype(np.float32) * s
                                      if bits > 8 else oracle.quantize(x, s, bits).astype(np.float32) * s)


def test_zero_sized_inputs():
    dx, dw, db = ste.ste_linear_backward(np.zeros((0, 3), np.float32), np.zeros((0, 5), np.float32), np.zeros((3, 5), np.float32), 1.0, 1.0, 8)
    assert dx.shape == (0, 5) and dw.shape == (3, 5) and not dw.any() and not db.any()


def test_sgd_step_hand_values_and_two_roundings():
    np.testing.assert_array_equal(ste.sgd_step([1.0, 2.0, -3.0], [0.5, -4.0, 0.25], 0.5), np.array([0.75, 4.0, -3.125], np.float32))
    # (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24 rounds (tie to even) to 1 + 2^-11: the difference is exactly 0 when the product is
    # rounded on its own, and -2^-24 if product and difference were fused
    a = np.float32(1 + 2.0 ** -12)
    assert ste.sgd_step([np.float32(1 + 2.0 ** -11)], [a], a)[0] == 0.0


@pytest.mark.parametrize("geo", [
    # N, C, H, W, O, kh, kw, stride, pad, dil
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 2, 9, 8, 3, 3, 2, (2, 1), (0, 1), (1, 2)),
    (3, 4, 6, 6, 2, 1, 1, (1, 1), (0, 0), (1, 1)),
    (2, 2, 10, 11, 3, 5, 3, (2, 3), (2, 1), (2, 1)),
])
def test_conv_backward_equals_autograd_of_fake_quantised_convolution(geo):
    import torch.nn.functional as F
    N, C, H, W, O, kh, kw, stride, pad, dil = geo
    bits, s_x, s_w = 6, 2.0 ** -3, 2.0 ** -5
    Q = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(sum(geo[:7]))
    x = (rng.integers(-4 * Q - 12, 4 * Q + 13, size=(N, C, H, W)) * 0.25 * s_x).astype(np.float32)
    w = (rng.integers(-4 * Q - 12, 4 * Q + 13, size=(O, C, kh, kw)) * 0.25 * s_w).astype(np.float32)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    bt = torch.zeros(O, dtype=torch.float64, requires_grad=True)

    def fq(t, s):
        r = t / s
        r = r + (torch.round(r) - r).detach()
        return torch.clamp(r, -Q, Q) * s

    y = F.conv2d(fq(xt, s_x), fq(wt, s_w), bt, stride, pad, dil)
    dy = rng.standard_normal(tuple(y.shape)).astype(np.float32)
    (y * torch.tensor(dy, dtype=torch.float64)).sum().backward()
    dx, dw, db = ste.ste_conv2d_backward(dy, x, w, stride, pad, dil, s_x, s_w, bits)
    assert (np.abs(x) > Q * s_x).any()
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-12, atol=1e-13)


def test_conv_backward_of_a_1x1_convolution_is_the_linear_backward():
    rng = np.random.default_rng(3)
    N, C, H, W, O, bits = 2, 5, 3, 4, 6, 8
    x = rng.standard_normal((N, C, H, W)).astype(np.float32); w = rng.standard_normal((O, C, 1, 1)).astype(np.float32) * 0.3
    dy = rng.standard_normal((N, O, H, W)).astype(np.float32)
    dx, dw, db = ste.ste_conv2d_backward(dy, x, w, (1, 1), (0, 0), (1, 1), 0.011, 0.004, bits)
    rows = lambda t: np.ascontiguousarray(np.transpose(t, (0, 2, 3, 1)).reshape(-1, t.shape[1]))
    lx, lw, lb = ste.ste_linear_backward(rows(dy), rows(x), w.reshape(O, C), 0.011, 0.004, bits)
    np.testing.assert_allclose(rows(dx), lx, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dw.reshape(O, C), lw, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(db, lb, rtol=1e-13)


def test_relu_backward_equals_autograd():
    v = np.array([-2.0, -0.0, 0.0, 1e-30, 3.0, np.nan], dtype=np.float32)
    dy = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0], dtype=np.float32)
    t = torch.tensor(v[:5], requires_grad=True)
    y = torch.relu(t)
    (y * torch.tensor(dy[:5])).sum().backward()
    got = ste.relu_backward(dy, np.maximum(v, 0))
    np.testing.assert_array_equal(got[:5], t.grad.numpy())
    np.testing.assert_array_equal(got[:5], [0, 0, 0, 4, 5])
