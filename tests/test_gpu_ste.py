"""GPU parity of the straight-through backward pass (Sec. III-A, "Retraining") against the CPU oracle, through the C ABI.

Tolerance.  The library forms every gradient element as an fp32 sum of R products of fp32 operands (matrix
instructions; any order).  For any order of an fp32 dot product of length R the error is at most
gamma(R + 1) * sum |a| |b| with gamma(n) = n u / (1 - n u), u = 2^-24; the oracle's fp64 sum is exact to 1e-16 of the
same quantity.  The clip mask and the fake-quantised operand values are decided in fp32 on both sides, so they
agree exactly: a masked element must be exactly 0.
"""
import numpy as np
import pytest
import torch

from oracle import ste

pytestmark = pytest.mark.gpu

U = 2.0 ** -24


@pytest.fixture(scope="module")
def B():
    from paper_2203_04071_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make(M, K, N, bits, seed, clip=1.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.1).astype(np.float32)
    dy = rng.standard_normal((M, N)).astype(np.float32)
    Q = (1 << (bits - 1)) - 1
    # scales from a clipping point below the maximum (as a percentile calibrator gives): some elements are clipped
    s_x = np.float32(clip * (np.abs(x).max() if x.size else 1.0) / Q)
    s_w = np.float32(clip * (np.abs(w).max() if w.size else 1.0) / Q)
    return dy, x, w, s_x, s_w


def check(got, want, bound, R):
    got = got.detach().cpu().numpy().astype(np.float64)
    assert got.shape == want.shape
    g = (R + 1) * U / (1 - (R + 1) * U)
    err = np.abs(got - want)
    assert (err <= g * bound + 1e-37).all(), f"max err/bound = {np.max(err / (g * bound + 1e-37))}"
    assert (got[want == 0] == 0).all()


CASES = [(1, 1, 1), (3, 5, 2), (64, 256, 128), (130, 129, 131), (257, 40, 300), (128, 128, 128), (300, 260, 17), (17, 1000, 33),
         (512, 16, 1), (1, 300, 513),
         # launch shapes of the larger products: 64-tiles with four waves (ragged, whole), 128-tiles with four waves (ragged,
         # whole) and with eight (ragged)
         (1600, 1300, 24), (1664, 1280, 32), (2100, 4100, 40), (2048, 4096, 64), (2000, 1700, 20)]


@pytest.mark.parametrize("bits,clip", [(8, 0.6), (4, 1.0), (12, 0.8)])
@pytest.mark.parametrize("M,K,N", CASES)
def test_ste_linear_backward_matches_oracle(B, M, K, N, bits, clip):
    dy, x, w, s_x, s_w = make(M, K, N, bits, M * 7 + K * 3 + N + bits, clip)
    if M * K > 4:
        x.flat[3] = np.nan                      # no gradient there; its fake-quantised value is 0
    if M * K > 40:                              # exact ties of the rounding and values around the clipping point
        Q = (1 << (bits - 1)) - 1
        x.flat[4:20] = (np.arange(16) - 8 + 0.5).astype(np.float32) * s_x
        x.flat[20:24] = np.array([Q + 0.5, -(Q + 0.5), Q, Q + 0.49], np.float32) * s_x
    dx, dw, db = B.adapt_ste_linear_backward_f32(dev(dy), dev(x), dev(w), s_x, s_w, bits)
    torch.cuda.synchronize()
    ox, ow, ob = ste.ste_linear_backward(dy, x, w, s_x, s_w, bits)
    bx, bw, bb = ste.ste_linear_backward_bound(dy, x, w, s_x, s_w, bits)
    if clip < 1.0 and M * K > 100:
        assert (ox == 0).sum() > 0 and (ow == 0).sum() > 0          # the mask is exercised
    check(dx, ox, bx, N)
    check(dw, ow, bw, M)
    check(db, ob, bb, M)


@pytest.mark.parametrize("M,K,N", [(0, 5, 3), (4, 0, 3), (4, 5, 0), (0, 0, 0)])
def test_ste_empty_dimensions(B, M, K, N):
    dy, x, w, s_x, s_w = make(M, K, N, 8, 1)
    dx, dw, db = B.adapt_ste_linear_backward_f32(dev(dy), dev(x), dev(w), 0.01, 0.01, 8)
    torch.cuda.synchronize()
    ox, ow, ob = ste.ste_linear_backward(dy, x, w, 0.01, 0.01, 8)
    np.testing.assert_array_equal(dx.cpu().numpy(), ox)
    np.testing.assert_array_equal(dw.cpu().numpy(), ow)             # M = 0: zeros, written
    check(db, ob, ste.ste_linear_backward_bound(dy, x, w, 0.01, 0.01, 8)[2], M)


def test_ste_unaligned_views_and_partial_outputs(B):
    # buffers that start 4 bytes past a 16-byte boundary take the element-wise loads; outputs left out are not touched
    M, K, N, bits = 70, 36, 44, 8
    dy, x, w, s_x, s_w = make(M, K, N, bits, 9, 0.7)
    def shifted(a):
        buf = torch.zeros(a.size + 1, dtype=torch.float32, device="cuda")
        buf[1:] = torch.from_numpy(a.ravel()).cuda()
        return buf[1:].view(a.shape)
    ox, ow, ob = ste.ste_linear_backward(dy, x, w, s_x, s_w, bits)
    bx, bw, bb = ste.ste_linear_backward_bound(dy, x, w, s_x, s_w, bits)
    dx, dw, db = B.adapt_ste_linear_backward_f32(shifted(dy), shifted(x), shifted(w), s_x, s_w, bits)
    torch.cuda.synchronize()
    check(dx, ox, bx, N); check(dw, ow, bw, M); check(db, ob, bb, M)
    dx, dw, db = B.adapt_ste_linear_backward_f32(dev(dy), dev(x), dev(w), s_x, s_w, bits, want=("dw",))
    assert dx is None and db is None
    check(dw, ow, bw, M)


def test_ste_full_size_projection_layer(B):
    # the input projection of the recurrent configuration: 6400 x 512 -> 2048, 7-bit operands, whole result compared
    M, K, N, bits = 6400, 512, 2048, 7
    dy, x, w, s_x, s_w = make(M, K, N, bits, 4, 0.5)
    dx, dw, db = B.adapt_ste_linear_backward_f32(dev(dy), dev(x), dev(w), s_x, s_w, bits)
    torch.cuda.synchronize()
    ox, ow, ob = ste.ste_linear_backward(dy, x, w, s_x, s_w, bits)
    bx, bw, bb = ste.ste_linear_backward_bound(dy, x, w, s_x, s_w, bits)
    check(dx, ox, bx, N); check(dw, ow, bw, M); check(db, ob, bb, M)
    # far inside the worst-case bound in practice: the typical error of an fp32 sum grows like sqrt(R)
    rel = np.abs(dx.cpu().numpy() - ox).max() / np.abs(ox).max()
    assert rel < 64 * U * np.sqrt(N)


def test_ste_refusals(B):
    dy, x, w, s_x, s_w = make(4, 8, 4, 8, 2)
    d = [dev(dy), dev(x), dev(w)]
    for kw in (dict(bits=1), dict(bits=17), dict(s_x=0.0), dict(s_w=float("nan")), dict(s_x=float("inf"))):
        a = dict(s_x=s_x, s_w=s_w, bits=8); a.update(kw)
        with pytest.raises(B.AdaptError) as e:
            B.adapt_ste_linear_backward_f32(d[0], d[1], d[2], a["s_x"], a["s_w"], a["bits"])
        assert e.value.code == -1
    L = B.load()
    import ctypes
    rc = L.adapt_ste_linear_backward_f32(d[0].data_ptr(), d[1].data_ptr(), d[2].data_ptr(), 4, 8, 4, ctypes.c_float(s_x), ctypes.c_float(s_w), 8,
                                         d[1].data_ptr(), None, None, None)           # dx aliases x
    assert rc == -1
    rc = L.adapt_ste_linear_backward_f32(None, d[1].data_ptr(), d[2].data_ptr(), 4, 8, 4, ctypes.c_float(s_x), ctypes.c_float(s_w), 8,
                                         None, d[0].data_ptr(), None, None)           # dy missing
    assert rc == -1


@pytest.mark.parametrize("n", [0, 1, 255, 4099, 1 << 21])
def test_sgd_step_bit_exact(B, n):
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32); g = rng.standard_normal(n).astype(np.float32)
    if n:
        a = np.float32(1 + 2.0 ** -12)
        w[0], g[0] = np.float32(1 + 2.0 ** -11), a          # exactly 0 with separate roundings at lr = a
    for lr in (np.float32(1 + 2.0 ** -12), np.float32(1e-4)):
        wd = dev(w)
        B.adapt_sgd_step_f32(wd, dev(g), lr)
        got = wd.cpu().numpy(); want = ste.sgd_step(w, g, lr)
        assert (got.view(np.uint32) == want.view(np.uint32)).all()


def test_retraining_loop_recovers_error_of_an_approximate_layer(B):
    """Forward through the multiplier table, straight-through backward, SGD: the loop of Sec. III-A on a synthetic
    regression task.  The student starts from perturbed weights; its loss through the approximate layer must fall
    well below the start and end near the floor set by 8-bit quantisation and the table's error."""
    from paper_2203_04071_amd import workloads as wl
    import oracle as orc
    rng = np.random.default_rng(11)
    M, K, N, bits = 256, 64, 32, 8
    x = rng.standard_normal((M, K)).astype(np.float32)
    w_true = (rng.standard_normal((N, K)) * 0.2).astype(np.float32)
    target = dev((x.astype(np.float64) @ w_true.astype(np.float64).T).astype(np.float32))
    w = dev((w_true + 0.1 * rng.standard_normal((N, K))).astype(np.float32))
    xd = dev(x)
    L = B.Lut(wl.make_lut(bits), bits)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    losses = []
    for it in range(40):
        s_w = orc.scale_from_amax(float(B.adapt_absmax_f32(w).item()), bits)
        pw = B.adapt_weights_pack_linear(L, B.adapt_quantize_f32(w, s_w, bits))
        y = B.adapt_linear_layer_f32(pw, xd, s_x, np.float32(s_x) * np.float32(s_w))
        diff = y - target
        losses.append(float((diff * diff).mean().item()))
        dy = (diff * (2.0 / diff.numel())).contiguous()
        _, dw, _ = B.adapt_ste_linear_backward_f32(dy, xd, w, s_x, s_w, bits, want=("dw",))
        B.adapt_sgd_step_f32(w, dw, 4.0)
        B.adapt_weights_destroy(pw)
    assert losses[-1] < 0.05 * losses[0], losses[::8]
    assert all(b < a * 1.05 for a, b in zip(losses, losses[1:])), losses       # no blow-up on the way


CONV_CASES = [
    # N, C, H, W, O, kh, kw, stride, pad, dil, bits
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1), (1, 1), 8),
    (1, 2, 9, 8, 3, 3, 2, (2, 1), (0, 1), (1, 2), 6),
    (3, 4, 6, 6, 2, 1, 1, (1, 1), (0, 0), (1, 1), 8),
    (2, 2, 10, 11, 3, 5, 3, (2, 3), (2, 1), (2, 1), 4),
    (8, 16, 16, 16, 32, 3, 3, (1, 1), (1, 1), (1, 1), 8),          # whole tiles: 2048 rows, 144 columns
    (4, 64, 32, 32, 64, 3, 3, (1, 1), (1, 1), (1, 1), 8),          # an eighth of the benchmark layer's batch
    (5, 13, 17, 19, 21, 3, 3, (2, 2), (1, 1), (1, 1), 7),          # nothing divides anything
    (16, 16, 32, 32, 16, 3, 3, (2, 2), (1, 1), (1, 1), 8),         # a stride-2 layer of the CNN configuration
    (0, 3, 5, 5, 2, 3, 3, (1, 1), (1, 1), (1, 1), 8),              # empty batch
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_ste_conv2d_backward_matches_oracle(B, case):
    """Same bar as the linear layer.  dw and db are fp32 sums of M = N Ho Wo terms in some fixed order (split into partial
    sums for small outputs): gamma(M + 1).  An element of dx is a sum of at most kh kw fp32 dot products of length Cout:
    gamma(Cout + kh kw + 1).  Both against the sums of absolute terms, which the oracle forms the same way."""
    N, C, H, W, O, kh, kw, stride, pad, dil, bits = case
    rng = np.random.default_rng(sum(case[:7]) + bits)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((O, C, kh, kw)) * 0.1).astype(np.float32)
    Ho = (H + 2 * pad[0] - dil[0] * (kh - 1) - 1) // stride[0] + 1
    Wo = (W + 2 * pad[1] - dil[1] * (kw - 1) - 1) // stride[1] + 1
    dy = rng.standard_normal((N, O, Ho, Wo)).astype(np.float32)
    Q = (1 << (bits - 1)) - 1
    s_x = np.float32(0.7 * (np.abs(x).max() if x.size else 1.0) / Q)
    s_w = np.float32(0.8 * np.abs(w).max() / Q)
    dx, dw, db = B.adapt_ste_conv2d_backward_f32(dev(dy), dev(x), dev(w), stride, pad, dil, s_x, s_w, bits)
    torch.cuda.synchronize()
    ox, ow, ob = ste.ste_conv2d_backward(dy, x, w, stride, pad, dil, s_x, s_w, bits)
    bx, bw, bb = ste.ste_conv2d_backward(dy, x, w, stride, pad, dil, s_x, s_w, bits, absolute=True)
    M = N * Ho * Wo
    if x.size > 100:
        assert (ox == 0).any() and (ow == 0).any()
    check(dx, ox, bx, O + kh * kw)
    check(dw, ow, bw, M)
    check(db, ob, bb, M)
    # only one of the gradients, with a workspace that is reused
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    dx2, dw2, db2 = B.adapt_ste_conv2d_backward_f32(dev(dy), dev(x), dev(w), stride, pad, dil, s_x, s_w, bits, want=("dx",), workspace=ws)
    assert dw2 is None and db2 is None and torch.equal(dx2, dx)


def test_ste_conv2d_refusals(B):
    import ctypes
    L = B.load()
    x = torch.zeros((2, 3, 8, 8), device="cuda"); w = torch.zeros((4, 3, 3, 3), device="cuda"); dy = torch.zeros((2, 4, 8, 8), device="cuda")
    dx = torch.empty_like(x)
    geo = (2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1)
    need = ctypes.c_size_t(0)
    assert L.adapt_ste_conv2d_backward_workspace(*geo, 1, 1, ctypes.byref(need)) == 0 and need.value > 0
    ws = torch.empty(need.value, dtype=torch.uint8, device="cuda")
    f = lambda wsp, nbytes, g=geo, bits=8: L.adapt_ste_conv2d_backward_f32(dy.data_ptr(), x.data_ptr(), w.data_ptr(), *g, ctypes.c_float(1.0),
                                                                          ctypes.c_float(1.0), bits, dx.data_ptr(), None, None, wsp, nbytes, None)
    assert f(ws.data_ptr(), need.value) == 0
    assert f(ws.data_ptr(), 16) == -1                      # too small
    assert f(None, need.value) == -1
    assert f(ws.data_ptr() + 4, need.value) == -1          # misaligned
    assert f(ws.data_ptr(), need.value, bits=1) == -1
    assert f(ws.data_ptr(), need.value, g=(2, 3, 2, 2, 4, 5, 5, 1, 1, 0, 0, 1, 1)) == -1       # filter larger than the image
    torch.cuda.synchronize()


def test_retraining_loop_of_an_approximate_convolution(B):
    """The same loop for a 3x3 convolution: forward through the table, straight-through backward over the unfolded input,
    SGD on the weights; the loss through the approximate layer must fall below a tenth of its start."""
    from paper_2203_04071_amd import workloads as wl
    import oracle as orc
    import torch.nn.functional as F
    rng = np.random.default_rng(12)
    N, C, HW, O, bits = 8, 8, 12, 8, 8
    x = rng.standard_normal((N, C, HW, HW)).astype(np.float32)
    w_true = (rng.standard_normal((O, C, 3, 3)) * 0.2).astype(np.float32)
    target = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w_true).double(), padding=1).float().cuda()
    w = dev((w_true + 0.1 * rng.standard_normal(w_true.shape)).astype(np.float32))
    xd = dev(x)
    L = B.Lut(wl.make_lut(bits), bits)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
    losses = []
    for it in range(60):
        s_w = orc.scale_from_amax(float(B.adapt_absmax_f32(w).item()), bits)
        pw = B.adapt_weights_pack_conv2d(L, B.adapt_quantize_f32(w, s_w, bits))
        y = B.adapt_conv2d_layer_f32(pw, xd, s_x, np.float32(s_x) * np.float32(s_w), (1, 1), (1, 1))
        diff = y - target
        losses.append(float((diff * diff).mean().item()))
        dy = (diff * (2.0 / diff.numel())).contiguous()
        _, dw, _ = B.adapt_ste_conv2d_backward_f32(dy, xd, w, (1, 1), (1, 1), (1, 1), s_x, s_w, bits, want=("dw",), workspace=ws)
        B.adapt_sgd_step_f32(w, dw, 1.0)
        B.adapt_weights_destroy(pw)
    assert losses[-1] < 0.1 * losses[0], losses[::10]
    assert max(losses[1:]) < losses[0], losses              # (near its floor the loss wanders with the rounding; it never blows up)


@pytest.mark.parametrize("n", [0, 1, 1000, (1 << 20) + 3])
def test_relu_backward_bit_exact(B, n):
    rng = np.random.default_rng(n + 5)
    y = np.maximum(rng.standard_normal(n), 0).astype(np.float32)
    dy = rng.standard_normal(n).astype(np.float32)
    if n >= 4:
        y[:4] = [0.0, -0.0, 1e-38, np.nan]
    want = ste.relu_backward(dy, y)
    got = B.adapt_relu_backward_f32(dev(dy), dev(y))
    assert (got.cpu().numpy().view(np.uint32) == want.view(np.uint32)).all()
    d = dev(dy)
    B.adapt_relu_backward_f32(d, dev(y), out=d)             # in place
    assert (d.cpu().numpy().view(np.uint32) == want.view(np.uint32)).all()


def test_retraining_loop_of_two_approximate_layers(B):
    """linear -> ReLU -> linear, both through the table: the second layer's input gradient goes through the ReLU gradient
    into the first layer's weight gradient, so the loop only converges if dx is a useful gradient too."""
    from paper_2203_04071_amd import workloads as wl
    import oracle as orc
    rng = np.random.default_rng(13)
    M, K1, Hd, N, bits = 256, 32, 48, 16, 8
    Q = (1 << (bits - 1)) - 1
    x = rng.standard_normal((M, K1)).astype(np.float32)
    w1_true = (rng.standard_normal((Hd, K1)) * 0.3).astype(np.float32)
    w2_true = (rng.standard_normal((N, Hd)) * 0.3).astype(np.float32)
    target = dev((np.maximum(x.astype(np.float64) @ w1_true.T, 0) @ w2_true.T).astype(np.float32))
    w1 = dev((w1_true + 0.08 * rng.standard_normal(w1_true.shape)).astype(np.float32))
    w2 = dev((w2_true + 0.08 * rng.standard_normal(w2_true.shape)).astype(np.float32))
    xd = dev(x)
    L = B.Lut(wl.make_lut(bits), bits)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    scale = lambda t: orc.scale_from_amax(float(B.adapt_absmax_f32(t).item()), bits)
    losses = []
    for it in range(80):
        s_w1, s_w2 = scale(w1), scale(w2)
        p1 = B.adapt_weights_pack_linear(L, B.adapt_quantize_f32(w1, s_w1, bits))
        p2 = B.adapt_weights_pack_linear(L, B.adapt_quantize_f32(w2, s_w2, bits))
        h = B.adapt_linear_layer_f32(p1, xd, s_x, np.float32(s_x) * np.float32(s_w1), act=B.ACT_RELU)
        s_h = scale(h)
        y = B.adapt_linear_layer_f32(p2, h, s_h, np.float32(s_h) * np.float32(s_w2))
        diff = y - target
        losses.append(float((diff * diff).mean().item()))
        dy = (diff * (2.0 / diff.numel())).contiguous()
        dh, dw2, _ = B.adapt_ste_linear_backward_f32(dy, h, w2, s_h, s_w2, bits, want=("dx", "dw"))
        B.adapt_relu_backward_f32(dh, h, out=dh)
        _, dw1, _ = B.adapt_ste_linear_backward_f32(dh, xd, w1, s_x, s_w1, bits, want=("dw",))
        B.adapt_sgd_step_f32(w1, dw1, 0.5)
        B.adapt_sgd_step_f32(w2, dw2, 0.5)
        B.adapt_weights_destroy(p1); B.adapt_weights_destroy(p2)
    assert np.isfinite(losses).all()
    assert losses[-1] < 0.3 * losses[0], losses[::10]
