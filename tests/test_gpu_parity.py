"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer results must be bit-exact; fp32 results within 1e-6 relative (they are in fact
produced by the same sequence of IEEE operations, and the elementwise tests check bit equality,
because one differing ulp before a quantiser would flip an integer downstream).
"""
import os

import numpy as np
import pytest
import torch

import oracle as orc
from oracle import networks as onet
from paper_2203_04071_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL = 1e-6


@pytest.fixture(scope="module")
def B():
    from paper_2203_04071_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def assert_f32_close(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape
    denom = np.maximum(np.abs(want), 1e-30)
    bad = np.abs(got - want) > RTOL * denom
    bad &= ~((got == 0) & (want == 0))
    assert not bad.any(), f"{bad.sum()} of {bad.size} differ; max rel {np.max(np.abs(got - want) / denom)}"


def bits_equal(a, b):
    a, b = np.ascontiguousarray(a, np.float32), np.ascontiguousarray(b, np.float32)
    return a.shape == b.shape and ((a.view(np.uint32) == b.view(np.uint32)) | ((a == 0) & (b == 0))).all()


def seeds(*base):
    """The seeds of a random-shape test: the fixed ones, plus ADAPT_EXTRA_SEEDS more (environment; default 0) for a longer
    campaign, e.g. ADAPT_EXTRA_SEEDS=200 python -m pytest tests -m gpu -k random."""
    extra = int(os.environ.get("ADAPT_EXTRA_SEEDS", "0"))
    return list(base) + [1000 * base[0] + i for i in range(extra)]


# ------------------------------------------------------------------ quantiser / dequantiser

@pytest.mark.parametrize("bits", [2, 4, 6, 7, 8])
@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4099, 1 << 20])
def test_quantize_bit_exact(B, bits, n):
    rng = np.random.default_rng(bits * 1000 + n % 997)
    x = (rng.standard_normal(n) * 3).astype(np.float32)
    if n >= 15:
        x[:7] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e30, -1e30]
        s0 = np.float32(0.37)
        x[7:15] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 4.5], np.float32) * s0   # ties
    for s in (np.float32(0.37), orc.scale_from_amax(orc.absmax(x[np.isfinite(x)]) if n else 0.0, bits)):
        got = host(B.adapt_quantize_f32(dev(x), s, bits)) if n else np.empty(0, np.int8)
        assert (got == orc.quantize(x, s, bits)).all()


def test_quantize_unaligned_pointers(B):
    rng = np.random.default_rng(5)
    x = rng.standard_normal(1000).astype(np.float32)
    xd = dev(x)
    out = torch.zeros(1003, dtype=torch.int8, device="cuda")
    B.adapt_quantize_f32(xd[1:], 0.05, 8, out=out[3:3 + 999])
    assert (host(out)[3:3 + 999] == orc.quantize(x[1:], 0.05, 8)).all()
    assert host(out)[:3].tolist() == [0, 0, 0] and host(out)[-1] == 0


@pytest.mark.parametrize("n", [0, 1, 5, 1023, 1 << 18, (1 << 20) + 3])
def test_absmax_exact(B, n):
    rng = np.random.default_rng(n % 1000)
    x = rng.standard_normal(n).astype(np.float32)
    if n > 4:
        x[3] = np.nan
        x[n // 2] = -7.25
    got = B.adapt_absmax_f32(dev(x)) if n else B.adapt_absmax_f32(torch.empty(0, device="cuda"))
    assert host(got)[0] == orc.absmax(x)


@pytest.mark.parametrize("shape", [(1, 1, 1), (5, 3, 7), (4, 16, 64), (64, 128, 1), (3, 10, 1), (2, 5, 12)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_dequant_bit_exact(B, shape, with_bias):
    rng = np.random.default_rng(sum(shape))
    acc = rng.integers(-2**31, 2**31 - 1, size=shape, dtype=np.int64).astype(np.int32)
    acc.reshape(-1)[0] = 2**24 + 1
    bias = rng.standard_normal(shape[1]).astype(np.float32) if with_bias else None
    s = np.float32(0.0123)
    want = orc.dequant(acc, s, *shape, bias)
    got = host(B.adapt_dequant_i32(dev(acc), s, *shape, dev(bias) if with_bias else None))
    assert bits_equal(got, want)
    assert_f32_close(got, want)


# ------------------------------------------------------------------ fp32 glue

def test_glue_ops_bit_exact(B):
    rng = np.random.default_rng(77)
    x = (rng.standard_normal((3, 5, 8, 8)) * 4).astype(np.float32)
    y = (rng.standard_normal((3, 5, 8, 8)) * 4).astype(np.float32)
    x[0, 0, 0, :3] = [np.nan, -0.0, 0.0]
    assert bits_equal(host(B.adapt_relu_f32(dev(x))), orc.relu(x))
    x[0, 0, 0, 0] = 1.0
    assert bits_equal(host(B.adapt_add_f32(dev(x), dev(y))), orc.add(x, y))
    assert bits_equal(host(B.adapt_add_f32(dev(x), dev(y), relu=True)), orc.relu(orc.add(x, y)))
    assert bits_equal(host(B.adapt_avgpool_hw_f32(dev(x))), orc.avgpool_hw(x))
    assert bits_equal(host(B.adapt_shortcut_a_f32(dev(x), 10)), orc.shortcut_a(x, 10))
    odd = (rng.standard_normal((2, 3, 7, 5))).astype(np.float32)
    assert bits_equal(host(B.adapt_shortcut_a_f32(dev(odd), 7)), orc.shortcut_a(odd, 7))
    v = np.concatenate([np.linspace(-100, 100, 100001), rng.standard_normal(100000) * 3,
                        [0.0, -0.0, 1e-30, -1e-30, 88.0, -87.0, 1e20]]).astype(np.float32)
    assert bits_equal(host(B.adapt_tanh_f32(dev(v))), orc.tanh(v))
    assert bits_equal(host(B.adapt_sigmoid_f32(dev(v))), orc.sigmoid(v))


@pytest.mark.parametrize("Bn,Hs", [(1, 1), (3, 17), (64, 512)])
def test_lstm_cell_bit_exact(B, Bn, Hs):
    rng = np.random.default_rng(Bn + Hs)
    a1 = rng.integers(-300000, 300000, size=(Bn, 4 * Hs)).astype(np.int32)
    a2 = rng.integers(-300000, 300000, size=(Bn, 4 * Hs)).astype(np.int32)
    bias = rng.standard_normal(4 * Hs).astype(np.float32)
    c = rng.standard_normal((Bn, Hs)).astype(np.float32)
    s1, s2 = np.float32(1.3e-5), np.float32(2.1e-5)
    for b in (bias, None):
        h_w, c_w = orc.lstm_cell(a1, a2, s1, s2, b, c)
        cd = dev(c)
        hd = torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
        B.adapt_lstm_cell_f32(dev(a1), dev(a2), s1, s2, dev(b) if b is not None else None, cd, hd)
        assert bits_equal(host(hd), h_w) and bits_equal(host(cd), c_w)
        # fused variant: same cell, plus the quantised h of the next step
        cd = dev(c)
        qd = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
        s_h = np.float32(1.0) / np.float32(63)
        B.adapt_lstm_cell_q_f32(dev(a1), dev(a2), s1, s2, dev(b) if b is not None else None, cd, hd, qd, s_h, 7)
        assert bits_equal(host(hd), h_w) and bits_equal(host(cd), c_w)
        assert (host(qd) == orc.quantize(h_w, s_h, 7)).all()


@pytest.mark.parametrize("Bn,Hs", [(1, 1), (3, 17), (64, 512)])
def test_gru_and_rnn_cells_bit_exact(B, Bn, Hs):
    rng = np.random.default_rng(7 + Bn + Hs)
    a1 = rng.integers(-300000, 300000, size=(Bn, 3 * Hs)).astype(np.int32)
    a2 = rng.integers(-300000, 300000, size=(Bn, 3 * Hs)).astype(np.int32)
    b1 = rng.standard_normal(3 * Hs).astype(np.float32)
    b2 = rng.standard_normal(3 * Hs).astype(np.float32)
    h = rng.uniform(-1, 1, (Bn, Hs)).astype(np.float32)
    s1, s2 = np.float32(1.3e-5), np.float32(2.1e-5)
    s_h = np.float32(1.0) / np.float32(63)
    for bi, bh in ((b1, b2), (None, b2), (b1, None), (None, None)):
        want = orc.gru_cell(a1, a2, s1, s2, bi, bh, h)
        hd = torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
        qd = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
        B.adapt_gru_cell_f32(dev(a1), dev(a2), s1, s2, dev(bi) if bi is not None else None, dev(bh) if bh is not None else None,
                             dev(h), hd, qd, s_h, 7)
        assert bits_equal(host(hd), want)
        assert (host(qd) == orc.quantize(want, s_h, 7)).all()
        hin = dev(h)                                            # in place, no quantised output
        B.adapt_gru_cell_f32(dev(a1), dev(a2), s1, s2, dev(bi) if bi is not None else None, dev(bh) if bh is not None else None,
                             hin, hin)
        assert bits_equal(host(hin), want)
    r1, r2, rb = a1[:, :Hs].copy(), a2[:, :Hs].copy(), b1[:Hs].copy()
    for relu in (False, True):
        for b in (rb, None):
            want = orc.rnn_cell(r1, r2, s1, s2, b, relu=relu)
            hd = torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
            qd = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
            B.adapt_rnn_cell_f32(dev(r1), dev(r2), s1, s2, dev(b) if b is not None else None, hd, relu, qd, s_h, 7)
            assert bits_equal(host(hd), want)
            assert (host(qd) == orc.quantize(want, s_h, 7)).all()


@pytest.mark.parametrize("kind", ["gru", "rnn"])
@pytest.mark.parametrize("bits", [7, 8])
def test_recurrent_layers_match_oracle(B, kind, bits):
    """GRU / plain recurrent layer end to end (quantise, input products, per-step hidden products, cells)."""
    from paper_2203_04071_amd import networks as gnet
    cfg = wl.recurrent_workload(kind, seq=12, batch=16, isz=96, hsz=72, bits=bits)
    want = onet.gru(cfg, threads=4) if kind == "gru" else onet.rnn(cfg, threads=4)
    net = gnet.Recurrent(cfg, kind, fused_step=False)               # product and cell as separate calls
    got = net.forward(dev(cfg["x"]))
    assert got["s_x"] == want["s_x"]
    assert (host(got["acc_ih"]) == want["acc_ih"]).all()
    assert (host(got["acc_hh_last"]) == want["acc_hh_last"]).all()
    assert bits_equal(host(got["hs"]), want["hs"])
    if True:                                                        # one kernel per time step
        net = gnet.Recurrent(cfg, kind)
        one = net.forward(dev(cfg["x"]))
        assert net.fused_step
        assert bits_equal(host(one["hs"]), want["hs"])


@pytest.mark.parametrize("shape", [(1, 2), (16, 72), (70, 130), (64, 512), (5, 6)])
@pytest.mark.parametrize("bits", [6, 8])
def test_gru_step_matches_product_and_cell(B, shape, bits):
    """The one-kernel GRU time step against the oracle's product followed by its cell, with and without biases, in place
    (h = h_prev) and out of place; odd hidden sizes are refused."""
    Bn, Hs = shape
    rng = np.random.default_rng(Bn * 1000 + Hs + bits)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    Q = (1 << (bits - 1)) - 1
    w_hh = wl.random_i8(rng, (3 * Hs, Hs), bits, "gauss")
    pw = B.adapt_weights_pack_linear(L, dev(w_hh))
    h_prev = np.tanh(rng.standard_normal((Bn, Hs))).astype(np.float32)
    s_h = np.float32(1.0) / np.float32(Q)
    qh = orc.quantize(h_prev, s_h, bits)
    acc_ih = rng.integers(-40000, 40000, size=(Bn, 3 * Hs)).astype(np.int32)
    acc_hh = orc.approx_linear(lut, bits, qh, w_hh, threads=4)
    s_ih, s_hh = np.float32(3e-5), np.float32(2e-5)
    b1 = rng.standard_normal(3 * Hs).astype(np.float32) * np.float32(0.2)
    b2 = rng.standard_normal(3 * Hs).astype(np.float32) * np.float32(0.2)
    for bi, bh in ((None, None), (b1, b2), (b1, None)):
        want = orc.gru_cell(acc_ih, acc_hh, s_ih, s_hh, bi, bh, h_prev)
        for inplace in (False, True):
            hp = dev(h_prev)
            hd = hp if inplace else torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
            qn = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
            B.adapt_gru_step_f32(pw, dev(qh), dev(acc_ih), s_ih, s_hh, s_h, dev(bi) if bi is not None else None,
                                 dev(bh) if bh is not None else None, hp, hd, qn)
            assert bits_equal(host(hd), want), (bi is not None, bh is not None, inplace)
            assert (host(qn) == orc.quantize(want, s_h, bits)).all()


@pytest.mark.parametrize("shape", [(1, 2), (16, 72), (70, 130), (64, 512)])
def test_rnn_step_matches_product_and_cell(B, shape):
    """The one-kernel plain recurrent step against the oracle's product followed by its cell (tanh and ReLU)."""
    Bn, Hs = shape
    bits = 7
    rng = np.random.default_rng(Bn * 1000 + Hs)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    Q = (1 << (bits - 1)) - 1
    w_hh = wl.random_i8(rng, (Hs, Hs), bits, "gauss")
    pw = B.adapt_weights_pack_linear(L, dev(w_hh))
    h_prev = np.tanh(rng.standard_normal((Bn, Hs))).astype(np.float32)
    s_h = np.float32(1.0) / np.float32(Q)
    qh = orc.quantize(h_prev, s_h, bits)
    acc_ih = rng.integers(-40000, 40000, size=(Bn, Hs)).astype(np.int32)
    acc_hh = orc.approx_linear(lut, bits, qh, w_hh, threads=4)
    s_ih, s_hh = np.float32(3e-5), np.float32(2e-5)
    b = rng.standard_normal(Hs).astype(np.float32) * np.float32(0.2)
    for bias, relu in ((None, False), (b, False), (b, True)):
        want = orc.rnn_cell(acc_ih, acc_hh, s_ih, s_hh, bias, relu=relu)
        hd = torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
        qn = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
        B.adapt_rnn_step_f32(pw, dev(qh), dev(acc_ih), s_ih, s_hh, s_h, dev(bias) if bias is not None else None, hd, qn, relu=relu)
        assert bits_equal(host(hd), want), (bias is not None, relu)
        assert (host(qn) == orc.quantize(want, s_h, bits)).all()
    if Hs == 2:
        pw3 = B.adapt_weights_pack_linear(L, dev(wl.random_i8(rng, (3, 3), bits)))
        z = lambda *s_, dt=torch.float32: torch.zeros(s_, dtype=dt, device="cuda")
        with pytest.raises(B.AdaptError) as e:      # odd hidden size
            B.adapt_rnn_step_f32(pw3, z(2, 3, dt=torch.int8), z(2, 3, dt=torch.int32), 1.0, 1.0, 1.0, None, z(2, 3), z(2, 3, dt=torch.int8))
        assert e.value.code == -2


def test_gru_step_refusals(B):
    L = B.Lut(wl.make_lut(7), 7)
    rng = np.random.default_rng(9)
    pw = B.adapt_weights_pack_linear(L, dev(wl.random_i8(rng, (9, 3), 7)))
    z = lambda *s_, dt=torch.float32: torch.zeros(s_, dtype=dt, device="cuda")
    with pytest.raises(B.AdaptError) as e:      # odd hidden size
        B.adapt_gru_step_f32(pw, z(2, 3, dt=torch.int8), z(2, 9, dt=torch.int32), 1.0, 1.0, 1.0, None, None, z(2, 3), z(2, 3), z(2, 3, dt=torch.int8))
    assert e.value.code == -2
    pw4 = B.adapt_weights_pack_linear(L, dev(wl.random_i8(rng, (16, 4), 7)))
    with pytest.raises(B.AdaptError) as e:      # a [4 Hs][Hs] handle
        B.adapt_gru_step_f32(pw4, z(2, 4, dt=torch.int8), z(2, 12, dt=torch.int32), 1.0, 1.0, 1.0, None, None, z(2, 4), z(2, 4), z(2, 4, dt=torch.int8))
    assert e.value.code == -1
    pw3 = B.adapt_weights_pack_linear(L, dev(wl.random_i8(rng, (12, 4), 7)))
    q = z(2, 4, dt=torch.int8)
    with pytest.raises(B.AdaptError) as e:      # aliasing operands
        B.adapt_gru_step_f32(pw3, q, z(2, 12, dt=torch.int32), 1.0, 1.0, 1.0, None, None, z(2, 4), z(2, 4), q)
    assert e.value.code == -1


# ------------------------------------------------------------------ table-lookup linear layer

LINEAR_SHAPES = [
    (1, 1, 1), (1, 7, 3), (3, 5, 17), (64, 256, 128), (65, 33, 9), (100, 64, 40), (130, 300, 24),
    (1000, 17, 5), (1025, 72, 16), (2500, 40, 33), (64, 512, 200), (7, 1000, 70),
]


@pytest.mark.parametrize("bits", [2, 5, 6, 7, 8])
@pytest.mark.parametrize("shape", LINEAR_SHAPES)
def test_linear_bit_exact(B, bits, shape):
    M, K, N = shape
    rng = np.random.default_rng(bits * 100000 + M * 31 + K * 7 + N)
    dist = "uniform" if (M + N) % 2 else "gauss"
    A = wl.random_i8(rng, (M, K), bits, dist)
    W = wl.random_i8(rng, (N, K), bits, dist)
    n = 1 << bits
    lut = rng.integers(-32768, 32768, size=(n, n)).astype(np.int32)     # arbitrary, asymmetric
    L = B.Lut(lut, bits)
    assert L.info()["storage"] == 0
    got = host(B.adapt_approx_linear(L, dev(A), dev(W)))
    assert (got == orc.approx_linear(lut, bits, A, W, threads=4)).all()


@pytest.mark.parametrize("bits", [4, 8])
def test_linear_wide_tables_and_wraparound(B, bits):
    """Entries beyond int16 use the two-half image; sums wrap modulo 2^32 like the oracle's."""
    rng = np.random.default_rng(bits)
    n = 1 << bits
    lut = rng.integers(-2**31, 2**31 - 1, size=(n, n), dtype=np.int64).astype(np.int32)
    L = B.Lut(lut, bits)
    assert L.info()["storage"] == 1 and L.info()["min"] == lut.min() and L.info()["max"] == lut.max()
    for (M, K, N) in [(70, 130, 20), (1100, 40, 9), (5, 600, 3)]:
        A = wl.random_i8(rng, (M, K), bits)
        W = wl.random_i8(rng, (N, K), bits)
        got = host(B.adapt_approx_linear(L, dev(A), dev(W)))
        assert (got == orc.approx_linear(lut, bits, A, W, threads=4)).all()
    x = wl.random_i8(rng, (2, 3, 6, 6), bits)
    w = wl.random_i8(rng, (4, 3, 3, 3), bits)
    assert (host(B.adapt_approx_conv2d(L, dev(x), dev(w), (1, 1), (1, 1))) == orc.approx_conv2d(lut, bits, x, w, (1, 1), (1, 1))).all()
    wt = wl.random_i8(rng, (3, 2, 4, 4), bits)
    assert (host(B.adapt_approx_conv_transpose2d(L, dev(x), dev(wt), 2, 1)) == orc.approx_conv_transpose2d(lut, bits, x, wt, 2, 1)).all()


def test_linear_empty_and_degenerate(B):
    lut = wl.make_lut(6)
    L = B.Lut(lut, 6)
    e = lambda *s: torch.empty(s, dtype=torch.int8, device="cuda")
    assert B.adapt_approx_linear(L, e(0, 8), e(4, 8)).shape == (0, 4)
    assert B.adapt_approx_linear(L, e(3, 8), e(0, 8)).shape == (3, 0)
    out = torch.full((3, 4), 99, dtype=torch.int32, device="cuda")
    B.adapt_approx_linear(L, e(3, 0), e(4, 0), out=out)          # K = 0: empty sums
    assert (host(out) == 0).all()
    # operands at both ends of the range, including -H which the quantiser itself never produces
    A = np.array([[-32, 31, 0, -32]], dtype=np.int8)
    W = np.array([[-32, -32, 31, 0], [31, 0, -32, -32]], dtype=np.int8)
    assert (host(B.adapt_approx_linear(L, dev(A), dev(W))) == orc.approx_linear(lut, 6, A, W)).all()


def test_linear_deterministic_and_overwrites(B):
    c = wl.config1()
    L = B.Lut(c["lut"], 8)
    A, W = dev(c["A"]), dev(c["W"])
    out = torch.full((64, 128), -1, dtype=torch.int32, device="cuda")
    B.adapt_approx_linear(L, A, W, out=out)
    first = host(out).copy()
    B.adapt_approx_linear(L, A, W, out=out)
    assert (host(out) == first).all()


def test_errors_on_device_handles(B):
    L = B.Lut(wl.make_lut(6), 6)
    x = torch.zeros((1, 4, 5, 5), dtype=torch.int8, device="cuda")
    w = torch.zeros((4, 2, 3, 3), dtype=torch.int8, device="cuda")
    w1 = torch.zeros((4, 4, 7, 7), dtype=torch.int8, device="cuda")
    dummy = torch.zeros((1, 4, 1, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(B.AdaptError) as e:
        B.adapt_approx_conv2d(L, x, w1, out=dummy)           # filter larger than the input
    assert e.value.code == -1
    with pytest.raises(B.AdaptError) as e:
        B.adapt_approx_conv2d(L, x, w, groups=3, out=dummy)         # channels not divisible by groups
    assert e.value.code == -1
    with pytest.raises(B.AdaptError):
        B.adapt_quantize_f32(torch.zeros(4, device="cuda"), -1.0, 8)


# ------------------------------------------------------------------ convolutions

CONV_CASES = [
    # N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw
    (2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 4, 9, 7, 6, 3, 3, 2, 2, 1, 1, 1, 1),
    (2, 2, 6, 10, 3, 1, 1, 1, 1, 0, 0, 1, 1),
    (1, 3, 7, 7, 2, 5, 3, 2, 1, 2, 0, 1, 1),
    (1, 4, 8, 8, 8, 3, 3, 1, 1, 2, 2, 2, 2),
    (1, 2, 4, 4, 3, 4, 4, 1, 1, 3, 3, 1, 1),
    (3, 16, 32, 32, 16, 3, 3, 1, 1, 1, 1, 1, 1),     # several row tiles, N = one channel tile
    (2, 16, 32, 32, 32, 3, 3, 2, 2, 1, 1, 1, 1),
    (5, 7, 13, 11, 19, 3, 3, 1, 1, 1, 1, 1, 1),      # ragged everything
    (1, 40, 6, 6, 70, 3, 3, 1, 1, 1, 1, 1, 1),       # short M, K split over waves
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw = case
    rng = np.random.default_rng(bits + sum(case))
    x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
    w = wl.random_i8(rng, (Cout, Cin, kh, kw), bits, "gauss")
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    got = host(B.adapt_approx_conv2d(L, dev(x), dev(w), (sh, sw), (ph, pw), (dh, dw)))
    want = orc.approx_conv2d(lut, bits, x, w, (sh, sw), (ph, pw), (dh, dw), threads=4)
    assert got.shape == want.shape and (got == want).all()


GROUPED_CASES = [
    # N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, groups
    (2, 6, 5, 5, 6, 3, 3, 1, 1, 1, 1, 1, 1, 6),            # depthwise
    (3, 32, 16, 16, 32, 3, 3, 1, 1, 1, 1, 1, 1, 32),       # depthwise, several workgroups
    (2, 24, 15, 13, 24, 5, 5, 2, 2, 2, 2, 1, 1, 24),       # depthwise 5x5 stride 2, ragged
    (2, 8, 9, 9, 16, 3, 3, 1, 1, 1, 1, 1, 1, 8),           # channel multiplier 2
    (1, 4, 8, 8, 8, 3, 3, 1, 1, 2, 2, 2, 2, 2),            # 2 groups of 2 -> 4, dilated
    (2, 12, 7, 7, 9, 3, 3, 1, 1, 1, 1, 1, 1, 3),           # 3 groups of 4 -> 3
    (2, 32, 12, 12, 64, 3, 3, 1, 1, 1, 1, 1, 1, 4),        # 4 groups of 8 -> 16: rows kernel, one launch over the groups
    (1, 48, 10, 10, 40, 3, 3, 2, 2, 1, 1, 1, 1, 2),        # 2 groups of 24 -> 20 (ragged channel tile)
    (3, 16, 33, 33, 16, 1, 1, 1, 1, 0, 0, 1, 1, 2),        # 1x1 grouped, 8 -> 8 per group
    (1, 8, 6, 210, 4, 5, 5, 1, 1, 2, 2, 1, 1, 2),          # wide rows: few output rows per tile
    (1, 8, 6, 900, 4, 5, 5, 1, 1, 2, 2, 1, 1, 2),          # input region of one output row too large to stage: direct form
    (2, 16, 20, 20, 16, 3, 3, 2, 2, 1, 1, 1, 1, 16),       # depthwise 3x3 stride 2
    (2, 10, 11, 9, 10, 5, 5, 1, 1, 2, 2, 1, 1, 10),        # depthwise 5x5, width not a multiple of 4
    (1, 6, 9, 14, 6, 3, 5, 1, 2, 1, 2, 1, 1, 6),           # 3x5 filter, horizontal stride 2
    (1, 6, 9, 14, 6, 3, 3, 1, 1, 1, 2, 1, 2, 6),           # horizontal dilation: pixel by pixel
    (2, 3, 70, 70, 3, 3, 3, 1, 1, 1, 1, 1, 1, 3),          # depthwise, planes larger than a tile: several row chunks
    (1, 64, 8, 8, 64, 3, 3, 1, 1, 1, 1, 1, 1, 64),         # small planes, many channels
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", GROUPED_CASES)
def test_grouped_conv2d_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, g = case
    rng = np.random.default_rng(bits + sum(case))
    x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
    w = wl.random_i8(rng, (Cout, Cin // g, kh, kw), bits, "gauss")
    lut = wl.make_lut(bits)
    got = host(B.adapt_approx_conv2d(B.Lut(lut, bits), dev(x), dev(w), (sh, sw), (ph, pw), (dh, dw), groups=g))
    want = orc.approx_conv2d(lut, bits, x, w, (sh, sw), (ph, pw), (dh, dw), g, threads=4)
    assert got.shape == want.shape and (got == want).all()


def test_grouped_conv2d_two_pass_table(B):
    """Entries beyond int16 (two table images, two passes) through both grouped paths."""
    rng = np.random.default_rng(77)
    lut = (rng.integers(-2**20, 2**20, size=(64, 64))).astype(np.int32)
    for (cin, cout, g) in ((8, 8, 8), (16, 32, 2)):
        x = wl.random_i8(rng, (2, cin, 9, 9), 6)
        w = wl.random_i8(rng, (cout, cin // g, 3, 3), 6)
        got = host(B.adapt_approx_conv2d(B.Lut(lut, 6), dev(x), dev(w), (1, 1), (1, 1), groups=g))
        assert (got == orc.approx_conv2d(lut, 6, x, w, (1, 1), (1, 1), (1, 1), g, threads=4)).all()


def test_separable_convolution_matches_oracle(B):
    """Eq. (1): depthwise then pointwise, each an approximate layer; calibrated and frozen-scale passes."""
    from paper_2203_04071_amd import networks as gnet
    cfg = wl.separable_workload()
    want = onet.separable_conv(cfg, threads=4)
    net = gnet.SeparableConv(cfg)
    got = net.forward(dev(cfg["x"]))
    assert [float(v) for v in got["scales"]] == [float(v) for v in want["scales"]]
    assert (host(got["acc_dw"]) == want["acc_dw"]).all()
    assert bits_equal(host(got["y"]), want["y"])
    assert bits_equal(host(got["out"]), want["out"])
    again = net.forward(dev(cfg["x"]), fused=False)             # frozen scales, separate steps
    assert bits_equal(host(again["out"]), want["out"])
    for keep_y in (True, False):                                # frozen scales, two kernels
        again = net.forward(dev(cfg["x"]), keep_y=keep_y)
        assert bits_equal(host(again["out"]), want["out"])
        if keep_y:
            assert bits_equal(host(again["y"]), want["y"])


def test_conv2d_padding_is_looked_up(B):
    c = 11
    t = np.full((16, 16), c, dtype=np.int32)
    rng = np.random.default_rng(5)
    x = wl.random_i8(rng, (2, 4, 5, 6), 4)
    w = wl.random_i8(rng, (3, 4, 3, 3), 4)
    got = host(B.adapt_approx_conv2d(B.Lut(t, 4), dev(x), dev(w), (1, 1), (1, 1)))
    assert (got == c * 4 * 9).all()


CONVT_CASES = [
    # N, Cin, H, W, Cout, k, stride, pad
    (2, 3, 1, 1, 4, 4, 1, 0),
    (1, 4, 4, 4, 3, 4, 2, 1),
    (2, 2, 5, 3, 2, 3, 2, 0),
    (1, 3, 3, 4, 2, 3, 1, 1),
    (1, 2, 4, 4, 2, 5, 3, 2),
    (3, 20, 8, 8, 12, 4, 2, 1),
    (2, 9, 16, 16, 3, 4, 2, 1),
    (70, 10, 1, 1, 24, 4, 1, 0),
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", CONVT_CASES)
def test_conv_transpose2d_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, k, s, p = case
    rng = np.random.default_rng(bits + sum(case))
    x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
    w = wl.random_i8(rng, (Cin, Cout, k, k), bits, "gauss")
    lut = wl.make_lut(bits)
    got = host(B.adapt_approx_conv_transpose2d(B.Lut(lut, bits), dev(x), dev(w), s, p))
    want = orc.approx_conv_transpose2d(lut, bits, x, w, s, p, threads=4)
    assert got.shape == want.shape and (got == want).all()


# ------------------------------------------------------------------ the five benchmark configurations

def test_config1_linear(B):
    c = wl.config1()
    L = B.Lut(c["lut"], 8)
    acc = B.adapt_approx_linear(L, dev(c["A"]), dev(c["W"]))
    want = orc.approx_linear(c["lut"], 8, c["A"], c["W"])
    assert (host(acc) == want).all()
    y = B.adapt_dequant_i32(acc, c["scale"], 64, 128, 1)
    assert_f32_close(host(y), orc.dequant(want, c["scale"], 64, 128, 1))
    # as bench.py times it: weights packed once, product on the packed handle
    pw = B.adapt_weights_pack_linear(L, dev(c["W"]))
    assert (host(B.adapt_approx_linear_packed(pw, dev(c["A"]))) == want).all()


@pytest.mark.parametrize("shape", [(64, 256, 128), (1, 64, 10), (130, 512, 24), (3000, 96, 40), (100, 100, 7), (64, 260, 16), (65, 1024, 130)])
@pytest.mark.parametrize("table", ["8-bit", "6-bit two-pass"])
def test_small_linear_layer_from_fp32(B, shape, table):
    """Linear layers below the streamed-table threshold as one call from fp32 activations (quantiser, whole-table product
    with the rescaling in its epilogue, or - two-pass table - a finishing pass): inner dimensions whose slices per lane
    are whole words and ones that are not (7 and 17 elements), a matrix on a 16-byte boundary and the same 4 bytes off
    it, ties of the quantiser.  The oracle's quantiser, product, rescaling, bias and ReLU, bit for bit."""
    M, K, N = shape
    rng = np.random.default_rng(M * 1000 + K + N)
    if table == "8-bit":
        bits = 8; lut = wl.make_lut(bits)
    else:
        bits = 6; lut = rng.integers(-2**20, 2**20, size=(64, 64)).astype(np.int32)
    L = B.Lut(lut, bits)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x.flat[:4] = np.array([0.5, 1.5, 2.5, -0.5], np.float32)[: min(4, x.size)]      # ties, once the scale is 1
    w = wl.random_i8(rng, (N, K), bits, "gauss")
    bias = rng.standard_normal(N).astype(np.float32)
    pw = B.adapt_weights_pack_linear(L, dev(w))
    for s_x in (orc.scale_from_amax(orc.absmax(x), bits), np.float32(1.0)):
        s_o = np.float32(s_x) * np.float32(0.01)
        acc = orc.approx_linear(lut, bits, orc.quantize(x, s_x, bits), w, threads=orc.host_threads())
        want = orc.relu(orc.dequant(acc, s_o, M, N, 1, bias)).reshape(M, N)
        got = host(B.adapt_linear_layer_f32(pw, dev(x), s_x, s_o, bias=dev(bias), act=B.ACT_RELU))
        assert bits_equal(got, want)
        # the same matrix 4 bytes off a 16-byte boundary
        buf = torch.empty(M * K + 1, dtype=torch.float32, device="cuda")
        xm = buf[1:].view(M, K)
        xm.copy_(dev(x))
        got = host(B.adapt_linear_layer_f32(pw, xm, s_x, s_o, bias=dev(bias), act=B.ACT_RELU))
        assert bits_equal(got, want)


def test_config2_conv_full_size(B):
    c = wl.config2()
    bits = 8
    th = orc.host_threads()
    x, w = dev(c["x"]), dev(c["w"])
    s_x = np.float32(host(B.adapt_absmax_f32(x))[0]) / np.float32(127)
    s_w = np.float32(host(B.adapt_absmax_f32(w))[0]) / np.float32(127)
    assert s_x == orc.scale_from_amax(orc.absmax(c["x"]), bits) and s_w == orc.scale_from_amax(orc.absmax(c["w"]), bits)
    qx, qw = B.adapt_quantize_f32(x, s_x, bits), B.adapt_quantize_f32(w, s_w, bits)
    oqx, oqw = orc.quantize(c["x"], s_x, bits), orc.quantize(c["w"], s_w, bits)
    assert (host(qx) == oqx).all() and (host(qw) == oqw).all()
    L = B.Lut(c["lut"], bits)
    acc = B.adapt_approx_conv2d(L, qx, qw, (1, 1), (1, 1))
    want = orc.approx_conv2d(c["lut"], bits, oqx, oqw, (1, 1), (1, 1), threads=th)
    assert (host(acc) == want).all()
    y = B.adapt_dequant_i32(acc, np.float32(s_x) * np.float32(s_w), 32, 64, 1024)
    assert_f32_close(host(y), orc.dequant(want, np.float32(s_x) * np.float32(s_w), 32, 64, 1024))


def test_config2_fused_layer_full_size_as_benchmarked(B):
    """The launch configuration bench.py times at config 2: one fused layer call on packed weights (quantise while the
    input is laid out, quad kernel, rescaling in its epilogue), whole tensor against the oracle."""
    c = wl.config2()
    bits = 8
    th = orc.host_threads()
    s_x = orc.scale_from_amax(orc.absmax(c["x"]), bits)
    s_w = orc.scale_from_amax(orc.absmax(c["w"]), bits)
    oqw = orc.quantize(c["w"], s_w, bits)
    want_acc = orc.approx_conv2d(c["lut"], bits, orc.quantize(c["x"], s_x, bits), oqw, (1, 1), (1, 1), threads=th)
    s_out = np.float32(s_x) * np.float32(s_w)
    want = orc.dequant(want_acc, s_out, 32, 64, 1024)
    L = B.Lut(c["lut"], bits)
    pw = B.adapt_weights_pack_conv2d(L, dev(oqw))
    x = dev(c["x"])
    for rep in range(2):
        got = host(B.adapt_conv2d_layer_f32(pw, x, s_x, s_out, (1, 1), (1, 1)))
        assert bits_equal(got.reshape(want.shape), want), rep
    assert (host(B.adapt_approx_conv2d_packed(pw, dev(orc.quantize(c["x"], s_x, bits)), (1, 1), (1, 1))) == want_acc).all()


def test_config3_resnet20_full_size(B):
    from paper_2203_04071_amd import networks as gnet
    c = wl.config3()
    th = orc.host_threads()
    want = onet.resnet20(c, threads=th, keep=True)
    net = gnet.ResNet20(c)
    keep = []
    got = net.forward(dev(c["x"]), keep=keep)
    assert [np.float32(s) for s in got["scales"]] == [np.float32(s) for s in want["scales"]]
    for i, (g, o) in enumerate(zip(keep, want["trace"])):
        assert (host(g) == o).all(), f"conv {i}"
    assert (host(got["fc_acc"]) == want["fc_acc"]).all()
    assert_f32_close(host(got["logits"]), want["logits"])
    again = net.forward(dev(c["x"]))                       # frozen scales: fused layer calls, no host reads
    assert bits_equal(host(again["logits"]), host(got["logits"]))
    assert bits_equal(host(again["feat"]), host(got["feat"]))
    assert_f32_close(host(again["feat"]), want["feat"])


def test_config4_lstm_full_size(B):
    from paper_2203_04071_amd import networks as gnet
    c = wl.config4()
    th = orc.host_threads()
    want = onet.lstm(c, threads=th)
    got = gnet.LSTM(c, fused_step=False).forward(dev(c["x"]))        # product and cell as separate calls
    assert np.float32(got["s_x"]) == np.float32(want["s_x"])
    assert (host(got["acc_ih"]) == want["acc_ih"]).all()
    assert (host(got["acc_hh_last"]) == want["acc_hh_last"]).all()
    net = gnet.LSTM(c)                                                # one kernel per time step
    one = net.forward(dev(c["x"]))
    assert net.fused_step, "the benchmark shape must fit the fused kernel"
    assert bits_equal(host(one["hs"]), want["hs"]) and bits_equal(host(one["c"]), want["c"])
    assert_f32_close(host(got["hs"]), want["hs"])
    assert_f32_close(host(got["c"]), want["c"])
    assert bits_equal(host(got["hs"]), want["hs"])          # the written-out gate functions make this exact


@pytest.mark.parametrize("bits", [6, 8])
def test_config5_dcgan_full_size(B, bits):
    from paper_2203_04071_amd import networks as gnet
    c = wl.config5(bits=bits)
    th = orc.host_threads()
    want = onet.dcgan(c, threads=th, keep=True)
    keep = []
    net = gnet.DCGAN(c)
    got = net.forward(dev(c["z"]), keep=keep)
    assert [np.float32(s) for s in got["scales"]] == [np.float32(s) for s in want["scales"]]
    for i, (g, o) in enumerate(zip(keep, want["accs"])):
        assert (host(g) == o).all(), f"layer {i}"
    assert_f32_close(host(got["out"]), want["out"])
    again = net.forward(dev(c["z"]))                        # frozen scales, layers chained: one kernel per layer after the first
    assert net.chain and net._chain_shape is not None, "the benchmark shapes must take the chained form"
    assert bits_equal(host(again["out"]), host(got["out"]))
    plain = gnet.DCGAN(c, chain=False)
    plain.scales = list(net.scales)
    assert bits_equal(host(plain.forward(dev(c["z"]))["out"]), host(got["out"]))       # one fused call per layer


# ------------------------------------------------------------------ long-matrix ("lines") kernel via packed weights

PACKED_LINEAR = [
    # M, K, N  (short products take the whole-table kernel with pre-packed offsets, long ones the derived-table kernel)
    (1, 8, 1), (5, 9, 3), (127, 32, 8), (129, 40, 9), (1024, 64, 16), (1500, 100, 20), (3000, 33, 7),
    (4100, 96, 24), (9000, 17, 65),
]


@pytest.mark.parametrize("bits", [2, 6, 7, 8])
@pytest.mark.parametrize("shape", PACKED_LINEAR)
def test_linear_packed_bit_exact(B, bits, shape):
    M, K, N = shape
    rng = np.random.default_rng(bits * 7919 + M + 3 * K + 5 * N)
    A = wl.random_i8(rng, (M, K), bits, "gauss" if M % 2 else "uniform")
    W = wl.random_i8(rng, (N, K), bits)
    n = 1 << bits
    lut = rng.integers(-32768, 32768, size=(n, n)).astype(np.int32)
    L = B.Lut(lut, bits)
    pw = B.adapt_weights_pack_linear(L, dev(W))
    got = host(B.adapt_approx_linear_packed(pw, dev(A)))
    assert (got == orc.approx_linear(lut, bits, A, W, threads=4)).all()


def test_linear_long_routes_through_lines_kernel_and_split_tables(B):
    rng = np.random.default_rng(99)
    for bits, wide in ((8, False), (8, True), (5, True)):
        n = 1 << bits
        lim = 2**31 - 1 if wide else 32767
        lut = rng.integers(-lim - 1, lim, size=(n, n), dtype=np.int64).astype(np.int32)
        L = B.Lut(lut, bits)
        for (M, K, N) in [(4096, 64, 8), (5000, 70, 19)]:
            A = wl.random_i8(rng, (M, K), bits)
            W = wl.random_i8(rng, (N, K), bits)
            want = orc.approx_linear(lut, bits, A, W, threads=4)
            assert (host(B.adapt_approx_linear(L, dev(A), dev(W))) == want).all()
            pw = B.adapt_weights_pack_linear(L, dev(W))
            assert (host(B.adapt_approx_linear_packed(pw, dev(A))) == want).all()


# Long linear layers: every variant of the derived-table kernel (rows per lane 8 / 4 / 2 by how many workgroups the
# shape gives on 256 compute units, regular or ragged row count, 8-bit or narrower index, signed or split table).
LINES_LINEAR = [
    (8192, 40, 256), (8197, 40, 256),        # 8 rows per lane
    (4096, 33, 256), (4099, 64, 250),        # 4 rows per lane
    (4096, 32, 16), (4101, 100, 9),          # 2 rows per lane
    (4096, 512, 16), (4101, 300, 9), (8192, 256, 64),      # long inner dimension, few tiles: split over workgroups
]


@pytest.mark.parametrize("kind", ["b8", "b8wide", "b6", "b5wide"])
@pytest.mark.parametrize("shape", LINES_LINEAR)
def test_linear_lines_kernel_variants(B, kind, shape):
    M, K, N = shape
    bits = {"b8": 8, "b8wide": 8, "b6": 6, "b5wide": 5}[kind]
    rng = np.random.default_rng(M + K + N + bits)
    if kind.endswith("wide"):
        n = 1 << bits
        lut = rng.integers(-2**31, 2**31 - 1, size=(n, n), dtype=np.int64).astype(np.int32)
    else:
        lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    A = wl.random_i8(rng, (M, K), bits, "gauss")
    W = wl.random_i8(rng, (N, K), bits)
    want = orc.approx_linear(lut, bits, A, W, threads=8)
    pw = B.adapt_weights_pack_linear(L, dev(W))
    got = host(B.adapt_approx_linear_packed(pw, dev(A)))
    assert (got == want).all()
    # short products with the same handle take the whole-table kernel with pre-packed offsets
    assert (host(B.adapt_approx_linear_packed(pw, dev(A[:37]))) == want[:37]).all()


PACKED_CONV = [
    # N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw
    (1, 8, 4, 4, 8, 3, 3, 1, 1, 1, 1, 1, 1),
    (2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 4, 9, 7, 6, 3, 3, 2, 2, 1, 1, 1, 1),
    (2, 2, 6, 10, 3, 1, 1, 1, 1, 0, 0, 1, 1),
    (1, 3, 7, 7, 2, 5, 3, 2, 1, 2, 0, 1, 1),
    (1, 4, 8, 8, 8, 3, 3, 1, 1, 2, 2, 2, 2),
    (3, 16, 32, 32, 16, 3, 3, 1, 1, 1, 1, 1, 1),
    (2, 16, 32, 32, 32, 3, 3, 2, 2, 1, 1, 1, 1),
    (5, 7, 13, 11, 19, 3, 3, 1, 1, 1, 1, 1, 1),
    (2, 40, 20, 20, 12, 3, 3, 1, 1, 1, 1, 1, 1),
    (8, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1, 1, 1),
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", PACKED_CONV)
def test_conv2d_packed_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw_, dh, dw = case
    rng = np.random.default_rng(bits + 17 * sum(case))
    x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
    w = wl.random_i8(rng, (Cout, Cin, kh, kw), bits, "gauss")
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    pk = B.adapt_weights_pack_conv2d(L, dev(w))
    got = host(B.adapt_approx_conv2d_packed(pk, dev(x), (sh, sw), (ph, pw_), (dh, dw)))
    want = orc.approx_conv2d(lut, bits, x, w, (sh, sw), (ph, pw_), (dh, dw), threads=8)
    assert got.shape == want.shape and (got == want).all()
    # plain entry point (routes by size) gives the same integers
    assert (host(B.adapt_approx_conv2d(L, dev(x), dev(w), (sh, sw), (ph, pw_), (dh, dw))) == want).all()


def test_packed_constant_table_counts_padding(B):
    t = np.full((16, 16), 7, dtype=np.int32)
    rng = np.random.default_rng(5)
    x = wl.random_i8(rng, (2, 5, 6, 6), 4)
    w = wl.random_i8(rng, (3, 5, 3, 3), 4)
    pk = B.adapt_weights_pack_conv2d(B.Lut(t, 4), dev(w))
    got = host(B.adapt_approx_conv2d_packed(pk, dev(x), (1, 1), (1, 1)))
    assert (got == 7 * 5 * 9).all()          # padded taps are looked up; padded channels/steps are not


def test_packed_handle_errors(B):
    L = B.Lut(wl.make_lut(6), 6)
    w = torch.zeros((4, 8), dtype=torch.int8, device="cuda")
    pw = B.adapt_weights_pack_linear(L, w)
    x = torch.zeros((1, 8, 5, 5), dtype=torch.int8, device="cuda")
    out = torch.zeros((1, 4, 5, 5), dtype=torch.int32, device="cuda")
    rc = B.load().adapt_approx_conv2d_packed(pw.handle, x.data_ptr(), out.data_ptr(), 1, 5, 5, 1, 1, 0, 0, 1, 1, None)
    assert rc == -1          # linear handle used for a convolution


# ------------------------------------------------------------------ transposed convolution, packed (phase form)

PACKED_CONVT = [
    # N, Cin, H, W, Cout, k, stride, pad
    (2, 8, 4, 4, 8, 4, 2, 1),          # generator geometry, 4 rows per image row (irregular rows)
    (3, 32, 8, 8, 16, 4, 2, 1),        # 8 regular rows per lane, fast kernel
    (2, 64, 16, 16, 24, 4, 2, 1),      # x-major activation copy
    (40, 32, 8, 8, 8, 4, 2, 1),
    (2, 5, 7, 5, 3, 4, 2, 1),          # ragged everything
    (1, 6, 5, 6, 4, 3, 1, 1),          # stride 1: one phase, borders on all sides
    (2, 4, 6, 6, 3, 3, 1, 0),
    (2, 4, 6, 6, 3, 3, 1, 2),
    (2, 7, 5, 5, 5, 2, 2, 0),          # kernel == stride: no overlap, no border terms
    (1, 4, 6, 4, 2, 4, 2, 0),
    (2, 4, 5, 5, 2, 4, 2, 2),          # crop wider than the border
    (1, 3, 4, 4, 2, 6, 2, 1),          # three taps per phase
    (1, 3, 4, 5, 2, 3, 3, 0),          # nine phases: more than one launch
    (1, 4, 4, 4, 2, 6, 3, 3),
    (2, 3, 5, 3, 2, 3, 2, 0),          # kernel no multiple of the stride: plain form inside the handle
    (1, 2, 4, 4, 2, 5, 3, 2),
    (4, 10, 1, 1, 6, 4, 1, 0),         # a single input pixel
    (3, 5, 1, 1, 2, 4, 2, 1),
    (300, 16, 4, 4, 8, 4, 2, 1),
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", PACKED_CONVT)
def test_conv_transpose2d_packed_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, k, s, p = case
    rng = np.random.default_rng(bits + 31 * sum(case))
    x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
    w = wl.random_i8(rng, (Cin, Cout, k, k), bits, "gauss")
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    want = orc.approx_conv_transpose2d(lut, bits, x, w, s, p, threads=8)
    pk = B.adapt_weights_pack_conv_transpose2d(L, dev(w), s)
    got = host(B.adapt_approx_conv_transpose2d_packed(pk, dev(x), p))
    assert got.shape == want.shape and (got == want).all()
    assert (host(B.adapt_approx_conv_transpose2d(L, dev(x), dev(w), s, p)) == want).all()


def test_conv_transpose2d_packed_rect_kernel_and_wide_table(B):
    # entries beyond int16 (two table halves) and a constant table: counts real pairs only
    rng = np.random.default_rng(77)
    bits = 5
    lut = rng.integers(-3_000_000, 3_000_000, size=(32, 32)).astype(np.int32)
    x = wl.random_i8(rng, (3, 9, 6, 8), bits)
    w = wl.random_i8(rng, (9, 5, 4, 4), bits)
    L = B.Lut(lut, bits)
    pk = B.adapt_weights_pack_conv_transpose2d(L, dev(w), 2)
    want = orc.approx_conv_transpose2d(lut, bits, x, w, 2, 1, threads=4)
    assert (host(B.adapt_approx_conv_transpose2d_packed(pk, dev(x), 1)) == want).all()
    t = np.full((16, 16), 3, dtype=np.int32)
    x = wl.random_i8(rng, (2, 4, 5, 5), 4)
    w = wl.random_i8(rng, (4, 3, 4, 4), 4)
    pk = B.adapt_weights_pack_conv_transpose2d(B.Lut(t, 4), dev(w), 2)
    got = host(B.adapt_approx_conv_transpose2d_packed(pk, dev(x), 1))
    # stride 2, kernel 4, pad 1: interior outputs meet 2 x 2 taps, edges 1 x 2, corners 1 x 1
    cnt = np.full((10, 10), 4)
    cnt[0, :] = cnt[-1, :] = cnt[:, 0] = cnt[:, -1] = 2
    cnt[0, 0] = cnt[0, -1] = cnt[-1, 0] = cnt[-1, -1] = 1
    assert (got == (3 * 4 * cnt)[None, None]).all()


# ------------------------------------------------------------------ LSTM time step in one kernel

@pytest.mark.parametrize("shape", [(1, 4, 6), (8, 16, 6), (64, 64, 7), (33, 100, 8), (64, 512, 7), (64, 512, 8), (150, 34, 7)])
def test_lstm_step_fused(B, shape):
    Bn, Hs, bits = shape
    rng = np.random.default_rng(sum(shape))
    lut = wl.make_lut(bits)
    W = wl.random_i8(rng, (4 * Hs, Hs), bits, "gauss")
    acc_ih = rng.integers(-40000, 40000, size=(Bn, 4 * Hs)).astype(np.int32)
    bias = rng.standard_normal(4 * Hs).astype(np.float32)
    qh = wl.random_i8(rng, (Bn, Hs), bits)
    c0 = rng.standard_normal((Bn, Hs)).astype(np.float32)
    Q = (1 << (bits - 1)) - 1
    s_h = np.float32(1.0) / np.float32(Q)
    s_ih, s_hh = np.float32(3e-5), np.float32(2e-4)
    acc_hh = orc.approx_linear(lut, bits, qh, W, threads=4)
    pw = B.adapt_weights_pack_linear(B.Lut(lut, bits), dev(W))
    for b in (bias, None):
        h_w, c_w = orc.lstm_cell(acc_ih, acc_hh, s_ih, s_hh, b, c0)
        cd = dev(c0)
        hd = torch.empty((Bn, Hs), dtype=torch.float32, device="cuda")
        qn = torch.empty((Bn, Hs), dtype=torch.int8, device="cuda")
        B.adapt_lstm_step_f32(pw, dev(qh), dev(acc_ih), s_ih, s_hh, s_h, dev(b) if b is not None else None, cd, hd, qn)
        assert bits_equal(host(hd), h_w) and bits_equal(host(cd), c_w)
        assert (host(qn) == orc.quantize(h_w, s_h, bits)).all()


def test_lstm_step_refuses_what_it_does_not_cover(B):
    L = B.Lut(wl.make_lut(6), 6)
    pw = B.adapt_weights_pack_linear(L, torch.zeros((4 * 5, 5), dtype=torch.int8, device="cuda"))     # odd Hs
    z = torch.zeros((3, 20), dtype=torch.int32, device="cuda")
    c = torch.zeros((3, 5), dtype=torch.float32, device="cuda")
    q = torch.zeros((3, 5), dtype=torch.int8, device="cuda")
    with pytest.raises(B.AdaptError) as e:
        B.adapt_lstm_step_f32(pw, q, z, 1.0, 1.0, 1.0, None, c, c.clone(), q.clone())
    assert e.value.code == -2


# ------------------------------------------------------------------ HIP-graph replay of a network

def test_graph_replay_matches_eager(B):
    """A recorded forward pass gives, on every replay (with eager work and synchronisations in between), exactly what
    the eager pass gives; checked on reduced sizes of the CNN, LSTM and generator configurations."""
    from paper_2203_04071_amd import networks as gnet
    c4 = wl.config4(seq=6, batch=8)
    c5 = wl.config5(bits=6, batch=8)
    c3 = wl.config3(batch=8)
    cases = [(gnet.ResNet20(c3), dev(c3["x"]), "logits"), (gnet.LSTM(c4), dev(c4["x"]), "hs"), (gnet.DCGAN(c5), dev(c5["z"]), "out")]
    for net, x, key in cases:
        want = host(net.forward(x)[key])            # calibrates
        assert bits_equal(host(net.forward(x)[key]), want)
        cap = gnet.Captured(net, x)
        for rep in range(3):
            got = cap.replay()[key]
            torch.cuda.synchronize()
            assert bits_equal(host(got), want), (type(net).__name__, rep)
            # eager work between replays, on other data
            other = host(net.forward(x * 0.5)[key])
            assert other.shape == want.shape
        # a different input through the same graph
        x2 = x * 0.75
        want2 = host(net.forward(x2)[key])
        assert bits_equal(host(cap.replay(x2)[key]), want2)


# ------------------------------------------------------------------ whole layers (fp32 in, fp32 out)

def _oracle_layer(acc, s_out, channels, inner, bias, act):
    outer = acc.size // (channels * inner)
    y = orc.dequant(acc, s_out, outer, channels, inner, bias)
    if act == 1:
        y = orc.relu(y)
    elif act == 2:
        y = orc.tanh(y)
    return y.reshape(acc.shape)


LAYER_LINEAR = [(37, 24, 10), (4096, 32, 16), (4101, 100, 9), (8192, 40, 256), (64, 512, 64)]


@pytest.mark.parametrize("kind", ["b8", "b6", "b5wide"])
@pytest.mark.parametrize("shape", LAYER_LINEAR)
def test_linear_layer_f32(B, kind, shape):
    M, K, N = shape
    bits = {"b8": 8, "b6": 6, "b5wide": 5}[kind]
    rng = np.random.default_rng(M + K + N + bits)
    lut = wl.make_lut(bits) if kind != "b5wide" else rng.integers(-2**31, 2**31 - 1, size=(32, 32), dtype=np.int64).astype(np.int32)
    x = rng.standard_normal((M, K)).astype(np.float32)
    W = wl.random_i8(rng, (N, K), bits)
    bias = rng.standard_normal(N).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    s_out = np.float32(s_x) * np.float32(0.013)
    acc = orc.approx_linear(lut, bits, orc.quantize(x, s_x, bits), W, threads=8)
    pw = B.adapt_weights_pack_linear(B.Lut(lut, bits), dev(W))
    for b, act in ((None, 0), (bias, 1), (bias, 2)):
        want = _oracle_layer(acc, s_out, N, 1, b, act)
        got = host(B.adapt_linear_layer_f32(pw, dev(x), s_x, s_out, dev(b) if b is not None else None, act))
        assert bits_equal(got, want), (b is not None, act)


LAYER_CONV = [
    # N, Cin, H, W, Cout, k, stride, pad
    (16, 64, 8, 8, 64, 3, 1, 1),       # few tiles, long inner dimension: split over workgroups
    (70, 32, 8, 8, 32, 3, 2, 1),
    (2, 3, 8, 8, 4, 3, 1, 1),
    (3, 16, 32, 32, 16, 3, 1, 1),
    (2, 16, 32, 32, 32, 3, 2, 1),
    (8, 64, 32, 32, 64, 3, 1, 1),
    (5, 7, 13, 11, 19, 3, 1, 1),
    (40, 32, 8, 8, 24, 3, 1, 1),
]


@pytest.mark.parametrize("kind", ["b8", "b6", "b5wide"])
@pytest.mark.parametrize("case", LAYER_CONV)
def test_conv2d_layer_f32(B, kind, case):
    N, Cin, H, W, Cout, k, st, pd = case
    bits = {"b8": 8, "b6": 6, "b5wide": 5}[kind]
    rng = np.random.default_rng(sum(case) + bits)
    lut = wl.make_lut(bits) if kind != "b5wide" else rng.integers(-2**31, 2**31 - 1, size=(32, 32), dtype=np.int64).astype(np.int32)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
    w = wl.random_i8(rng, (Cout, Cin, k, k), bits, "gauss")
    bias = rng.standard_normal(Cout).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    s_out = np.float32(s_x) * np.float32(0.02)
    acc = orc.approx_conv2d(lut, bits, orc.quantize(x, s_x, bits), w, (st, st), (pd, pd), threads=8)
    pw = B.adapt_weights_pack_conv2d(B.Lut(lut, bits), dev(w))
    for b, act in ((None, 0), (bias, 1), (None, 2)):
        want = _oracle_layer(acc, s_out, Cout, acc.shape[2] * acc.shape[3], b, act)
        got = host(B.adapt_conv2d_layer_f32(pw, dev(x), s_x, s_out, (st, st), (pd, pd), (1, 1), dev(b) if b is not None else None, act))
        assert bits_equal(got, want), (b is not None, act)
    # residual input: y = act((float(acc) * s + bias) + residual)
    res = rng.standard_normal(acc.shape).astype(np.float32)
    for b, act in ((None, 0), (bias, 1)):
        y = orc.add(orc.dequant(acc, s_out, N, Cout, acc.shape[2] * acc.shape[3], b), res)
        want = (orc.relu(y) if act == 1 else y).reshape(acc.shape)
        got = host(B.adapt_conv2d_layer_f32(pw, dev(x), s_x, s_out, (st, st), (pd, pd), (1, 1), dev(b) if b is not None else None, act,
                                            residual=dev(res)))
        assert bits_equal(got, want), ("residual", b is not None, act)


LAYER_CONVT = [
    (2, 8, 4, 4, 8, 4, 2, 1),
    (3, 32, 8, 8, 16, 4, 2, 1),
    (2, 64, 16, 16, 24, 4, 2, 1),
    (2, 7, 5, 5, 5, 2, 2, 0),          # no border terms: rescaled inside the product kernel
    (2, 3, 5, 3, 2, 3, 2, 0),          # plain form
    (4, 10, 1, 1, 6, 4, 1, 0),         # single input pixel
    # big-layer kernel, 4 rows per row slot; channel tiles that share an XCD between several row tiles:
    (64, 32, 16, 16, 32, 4, 2, 1),     # 4 channel tiles, 16 row tiles per phase: the phases of a row tile stay on one XCD
    (60, 32, 16, 16, 32, 4, 2, 1),     # 15 row tiles: the plain phase-fastest order
    (256, 16, 16, 16, 8, 4, 2, 1),     # 1 channel tile, 64 row tiles
    (252, 16, 16, 16, 5, 4, 2, 1),     # 63 row tiles, 5 of 8 channels
]


@pytest.mark.parametrize("kind", ["b8", "b6", "b5wide"])
@pytest.mark.parametrize("case", LAYER_CONVT)
def test_conv_transpose2d_layer_f32(B, kind, case):
    N, Cin, H, W, Cout, k, st, pd = case
    bits = {"b8": 8, "b6": 6, "b5wide": 5}[kind]
    rng = np.random.default_rng(sum(case) + bits)
    lut = wl.make_lut(bits) if kind != "b5wide" else rng.integers(-2**31, 2**31 - 1, size=(32, 32), dtype=np.int64).astype(np.int32)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
    w = wl.random_i8(rng, (Cin, Cout, k, k), bits, "gauss")
    bias = rng.standard_normal(Cout).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    s_out = np.float32(s_x) * np.float32(0.02)
    acc = orc.approx_conv_transpose2d(lut, bits, orc.quantize(x, s_x, bits), w, st, pd, threads=8)
    pw = B.adapt_weights_pack_conv_transpose2d(B.Lut(lut, bits), dev(w), st)
    for b, act in ((None, 0), (bias, 1), (bias, 2)):
        want = _oracle_layer(acc, s_out, Cout, acc.shape[2] * acc.shape[3], b, act)
        got = host(B.adapt_conv_transpose2d_layer_f32(pw, dev(x), s_x, s_out, pd, dev(b) if b is not None else None, act))
        assert bits_equal(got, want), (b is not None, act)


# ------------------------------------------------------------------ per-channel ranges, percentile calibrator

@pytest.mark.parametrize("shape", [(1, 1), (7, 45), (64, 576), (130, 1), (3, 5000)])
def test_per_channel_quantiser_bit_exact(B, shape):
    rows, cols = shape
    rng = np.random.default_rng(rows * 31 + cols)
    w = (rng.standard_normal((rows, cols)) * rng.uniform(0.01, 3.0, size=(rows, 1))).astype(np.float32)
    if rows > 2:
        w[1] = 0
    amax = host(B.adapt_absmax_rows_f32(dev(w)))
    assert bits_equal(amax, orc.absmax_rows(w))
    for bits in (4, 8):
        scales = np.array([orc.scale_from_amax(a, bits) for a in amax], dtype=np.float32)
        q = host(B.adapt_quantize_rows_f32(dev(w), dev(scales), bits))
        assert (q == orc.quantize_rows(w, scales, bits)).all()


@pytest.mark.parametrize("shape", [(1, 1, 1), (5, 3, 7), (4, 16, 64), (64, 128, 1)])
def test_per_channel_dequant_bit_exact(B, shape):
    o, c, i = shape
    rng = np.random.default_rng(sum(shape))
    acc = rng.integers(-2**31, 2**31 - 1, size=shape, dtype=np.int64).astype(np.int32)
    s = rng.uniform(1e-6, 1e-2, size=c).astype(np.float32)
    b = rng.standard_normal(c).astype(np.float32)
    for bias in (None, b):
        got = host(B.adapt_dequant_i32_per_channel(dev(acc), dev(s), o, c, i, dev(bias) if bias is not None else None))
        assert bits_equal(got, orc.dequant_per_channel(acc, s, o, c, i, bias))


@pytest.mark.parametrize("n,bins", [(1, 1), (1000, 8), (100_003, 2048), (1 << 20, 4096), (5000, 100)])
def test_histogram_and_percentile_bit_exact(B, n, bins):
    rng = np.random.default_rng(n + bins)
    x = (rng.standard_normal(n) ** 3).astype(np.float32)
    if n > 10:
        x[3] = np.nan
    amax = orc.absmax(np.nan_to_num(x))
    if not amax > 0:
        amax = np.float32(1.0)
    want = orc.histogram_abs(x, amax, bins)
    counts = B.adapt_histogram_abs_f32(dev(x), amax, bins)
    assert (host(counts).view(np.uint32) == want).all()
    # a second batch accumulates into the same counters
    y = (rng.standard_normal(n // 2 + 1) * np.float32(0.3) * amax).astype(np.float32)
    want2 = orc.histogram_abs(y, amax, bins, want.copy())
    B.adapt_histogram_abs_f32(dev(y), amax, bins, counts)
    assert (host(counts).view(np.uint32) == want2).all()
    for num, den in ((999, 1000), (1, 2), (1000, 1000), (0, 7)):
        got = host(B.adapt_percentile_from_histogram(counts, amax, num, den))[0]
        assert np.float32(got) == orc.percentile_from_histogram(want2, amax, num, den), (num, den)
    if bins <= 2048:        # (the oracle's search is quadratic in the bins)
        for bits in (4, 8, 12):
            got = host(B.adapt_mse_from_histogram(counts, amax, bits))[0]
            assert np.float32(got) == orc.mse_from_histogram(want2, amax, bits), bits
    for bits in (4, 8, 12):
        check_entropy_choice(B, counts, want2, amax, bits)


def check_entropy_choice(B, counts_dev, counts, amax, bits):
    """The information-loss calibrator picks the oracle's range; the two sides use different fp64 logarithm routines (last
    digit may differ), so when the picks differ the oracle's loss at the kernel's pick must equal its minimum to 1e-12."""
    got = np.float32(host(B.adapt_entropy_from_histogram(counts_dev, amax, bits))[0])
    want, kl = orc.entropy_from_histogram(counts, amax, bits, with_losses=True)
    if got == want:
        return
    bins = counts.size
    width = np.float32(np.float32(amax) / np.float32(bins))
    k = int(round(float(got) / float(width)))
    assert 1 <= k <= bins and np.float32(np.float32(k) * width) == got, (got, want)
    assert np.isfinite(kl[k - 1]) and abs(kl[k - 1] - np.min(kl)) <= 1e-12 * max(1.0, abs(np.min(kl))), (k, kl[k - 1], np.min(kl))


@pytest.mark.parametrize("case", ["flat", "ended", "empty", "outlier", "few_bins", "hand"])
def test_entropy_calibrator_special_histograms(B, case):
    bits, bins, amax = 4, 64, np.float32(3.2)
    rng = np.random.default_rng(5)
    counts = np.full(bins, 5, np.uint32)
    if case == "ended":
        counts[24:] = 0
    elif case == "empty":
        counts[:] = 0
    elif case == "outlier":
        counts = ((rng.integers(0, 9, bins) + 1) * 100).astype(np.uint32)
        counts[40:] = 0
        counts[63] = 1
    elif case == "few_bins":
        counts, bits, amax = np.array([3, 1, 2], np.uint32), 8, np.float32(6.0)
    elif case == "hand":
        counts, bits, amax = np.array([4, 2, 1, 1], np.uint32), 2, np.float32(4.0)
    got = np.float32(host(B.adapt_entropy_from_histogram(dev(counts.view(np.int32)), amax, bits))[0])
    assert got == orc.entropy_from_histogram(counts, amax, bits), case


def test_conv_layer_with_per_channel_weights_and_percentile_activations(B):
    """The paper's calibration recipe end to end on one layer: activation range from the 99.9 % histogram percentile,
    weight ranges per output channel, 8-bit table; integers and rescaled outputs against the oracle."""
    rng = np.random.default_rng(2024)
    bits, bins = 8, 2048
    x = (rng.standard_normal((4, 16, 12, 12)) ** 3).astype(np.float32)
    w = (rng.standard_normal((24, 16, 3, 3)) * rng.uniform(0.05, 2.0, size=(24, 1, 1, 1))).astype(np.float32)
    lut = wl.make_lut(bits)
    # oracle side
    amax = orc.absmax(x)
    cmax = orc.percentile_from_histogram(orc.histogram_abs(x, amax, bins), amax)
    s_x = orc.scale_from_amax(cmax, bits)
    s_w = np.array([orc.scale_from_amax(a, bits) for a in orc.absmax_rows(w)], dtype=np.float32)
    oqx, oqw = orc.quantize(x, s_x, bits), orc.quantize_rows(w, s_w, bits)
    acc_w = orc.approx_conv2d(lut, bits, oqx, oqw, (1, 1), (1, 1), threads=4)
    s_out = (np.float32(s_x) * s_w).astype(np.float32)
    want = orc.dequant_per_channel(acc_w, s_out, 4, 24, 144)
    # library side
    xd, wd = dev(x), dev(w)
    amax_g = np.float32(host(B.adapt_absmax_f32(xd))[0])
    cmax_g = np.float32(host(B.adapt_percentile_from_histogram(B.adapt_histogram_abs_f32(xd, amax_g, bins), amax_g))[0])
    assert amax_g == amax and cmax_g == cmax and cmax < amax
    sw_g = np.array([orc.scale_from_amax(a, bits) for a in host(B.adapt_absmax_rows_f32(wd))], dtype=np.float32)
    assert bits_equal(sw_g, s_w)
    qx = B.adapt_quantize_f32(xd, s_x, bits)
    qw = B.adapt_quantize_rows_f32(wd, dev(s_w), bits)
    assert (host(qx) == oqx).all() and (host(qw) == oqw).all()
    acc = B.adapt_approx_conv2d_packed(B.adapt_weights_pack_conv2d(B.Lut(lut, bits), qw), qx, (1, 1), (1, 1))
    assert (host(acc) == acc_w).all()
    y = B.adapt_dequant_i32_per_channel(acc, dev(s_out), 4, 24, 144)
    assert bits_equal(host(y), want)
    # and as one fused layer call with the vector of output scales (+ bias, ReLU)
    bias = rng.standard_normal(24).astype(np.float32)
    pw = B.adapt_weights_pack_conv2d(B.Lut(lut, bits), qw)
    y2 = B.adapt_conv2d_layer_f32(pw, xd, s_x, dev(s_out), (1, 1), (1, 1), bias=dev(bias), act=B.ACT_RELU)
    assert bits_equal(host(y2), orc.relu(orc.dequant_per_channel(acc_w, s_out, 4, 24, 144, bias)))
    # a long linear layer and a transposed convolution take the same vector
    Wl = (rng.standard_normal((24, 64)) * rng.uniform(0.05, 2.0, size=(24, 1))).astype(np.float32)
    xl = rng.standard_normal((4200, 64)).astype(np.float32)
    swl = np.array([orc.scale_from_amax(a, bits) for a in orc.absmax_rows(Wl)], dtype=np.float32)
    sxl = orc.scale_from_amax(orc.absmax(xl), bits)
    oql = orc.quantize_rows(Wl, swl, bits)
    accl = orc.approx_linear(lut, bits, orc.quantize(xl, sxl, bits), oql, threads=4)
    sol = (np.float32(sxl) * swl).astype(np.float32)
    yl = B.adapt_linear_layer_f32(B.adapt_weights_pack_linear(B.Lut(lut, bits), dev(oql)), dev(xl), sxl, dev(sol))
    assert bits_equal(host(yl), orc.dequant_per_channel(accl, sol, 4200, 24, 1))
    wt = wl.random_i8(rng, (16, 24, 4, 4), bits, "gauss")
    acct = orc.approx_conv_transpose2d(lut, bits, oqx, wt, 2, 1, threads=4)
    yt = B.adapt_conv_transpose2d_layer_f32(B.adapt_weights_pack_conv_transpose2d(B.Lut(lut, bits), dev(wt), 2), xd, s_x, dev(s_out), 1,
                                            bias=dev(bias), act=B.ACT_TANH)
    assert bits_equal(host(yt), orc.tanh(orc.dequant_per_channel(acct, s_out, 4, 24, 24 * 24, bias)))


# ------------------------------------------------------------------ operands wider than 8 bits, multipliers as functions

def _rand_i16(rng, shape, bits, dist="gauss"):
    h = 1 << (bits - 1)
    if dist == "uniform":
        return rng.integers(-h, h, size=shape).astype(np.int16)
    return np.clip(np.rint(rng.standard_normal(shape) * (h / 5.2)), -h, h - 1).astype(np.int16)


def test_quantize_i16_bit_exact(B):
    rng = np.random.default_rng(50)
    x = np.concatenate([rng.standard_normal(100003) * 3, [0.0, -0.0, 0.5, 1.5, 2.5, -2.5, 1e30, -1e30, np.nan, np.inf]]).astype(np.float32)
    for bits, s in ((12, 0.0031), (16, 1e-4), (8, 0.05), (2, 1.0)):
        got = host(B.adapt_quantize_i16_f32(dev(x), s, bits))
        assert (got == orc.quantize_i16(x, s, bits)).all()


BIG_LINEAR = [(1, 1, 1), (64, 256, 128), (300, 77, 19), (1025, 40, 8), (5, 0, 3)]


@pytest.mark.parametrize("bits", [9, 12])
@pytest.mark.parametrize("shape", BIG_LINEAR)
def test_linear_i16_table_bit_exact(B, bits, shape):
    M, K, N = shape
    rng = np.random.default_rng(bits + sum(shape))
    lut = wl.make_lut(bits)
    L = B.Lut16(bits, table=lut)
    for dist in ("gauss", "uniform"):
        a = _rand_i16(rng, (M, K), bits, dist)
        w = _rand_i16(rng, (N, K), bits, dist)
        got = host(B.adapt_approx_linear_i16(L, dev(a), dev(w)))
        assert (got == orc.approx_linear_i16(lut, bits, a, w, threads=4)).all()


BIG_CONV = [
    # N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw
    (2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 5, 9, 7, 11, 3, 3, 2, 2, 1, 1, 1, 1),
    (3, 16, 20, 20, 16, 3, 3, 1, 1, 1, 1, 1, 1),
    (1, 4, 8, 8, 8, 3, 3, 1, 1, 2, 2, 2, 2),
    (2, 6, 6, 10, 3, 1, 1, 1, 1, 0, 0, 1, 1),
]


@pytest.mark.parametrize("bits", [10, 12])
@pytest.mark.parametrize("case", BIG_CONV)
def test_conv2d_i16_table_bit_exact(B, bits, case):
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw = case
    rng = np.random.default_rng(bits + sum(case))
    lut = wl.make_lut(bits)
    x = _rand_i16(rng, (N, Cin, H, W), bits)
    w = _rand_i16(rng, (Cout, Cin, kh, kw), bits)
    got = host(B.adapt_approx_conv2d_i16(B.Lut16(bits, table=lut), dev(x), dev(w), (sh, sw), (ph, pw), (dh, dw)))
    want = orc.approx_conv2d_i16(bits, x, w, lut=lut, stride=(sh, sw), pad=(ph, pw), dil=(dh, dw), threads=4)
    assert got.shape == want.shape and (got == want).all()


@pytest.mark.parametrize("kind,param,bits", [(0, 0, 16), (1, 3, 12), (2, 0, 12), (2, 0, 16), (1, 1, 8), (2, 0, 5)])
def test_function_multipliers_bit_exact(B, kind, param, bits):
    rng = np.random.default_rng(kind * 100 + bits)
    a = _rand_i16(rng, (130, 96), bits, "uniform")
    w = _rand_i16(rng, (21, 96), bits, "uniform")
    got = host(B.adapt_approx_linear_func_i16(kind, param, bits, dev(a), dev(w)))
    assert (got == orc.approx_linear_func_i16(kind, param, bits, a, w, threads=4)).all()
    x = _rand_i16(rng, (2, 5, 9, 8), bits)
    f = _rand_i16(rng, (7, 5, 3, 3), bits)
    got = host(B.adapt_approx_conv2d_func_i16(kind, param, bits, dev(x), dev(f), (1, 1), (1, 1)))
    assert (got == orc.approx_conv2d_i16(bits, x, f, func=(kind, param), pad=(1, 1), threads=4)).all()
    if bits <= 12:
        # the table generated on the device from the function gives the same sums (and equals the oracle's table)
        L = B.Lut16(bits, func=(kind, param))
        assert (host(B.adapt_approx_linear_i16(L, dev(a), dev(w))) ==
                orc.approx_linear_i16(orc.table_from_func(kind, param, bits), bits, a, w, threads=4)).all()


@pytest.mark.parametrize("form", ["table12", "table9", "mitchell14", "trunc16"])
def test_i16_whole_layers_match_oracle_steps(B, form):
    """Whole layers on operands beyond 8 bits (quantise + product + rescale, bias, activation in one call) against the
    oracle's separate steps, table and function forms, scalar and per-channel scales, the three activations."""
    rng = np.random.default_rng(len(form) * 7 + 1)
    if form.startswith("table"):
        bits = int(form[5:])
        lut = orc.table_from_func(2 if bits == 12 else 1, 0 if bits == 12 else 3, bits)
        mul = B.Lut16(bits, table=lut)
        lin = lambda a, w: orc.approx_linear_i16(lut, bits, a, w, threads=4)
        conv = lambda x, w, **kw: orc.approx_conv2d_i16(bits, x, w, lut=lut, threads=4, **kw)
    else:
        kind, param, bits = (2, 0, 14) if form == "mitchell14" else (1, 5, 16)
        mul = (kind, param, bits)
        lin = lambda a, w: orc.approx_linear_func_i16(kind, param, bits, a, w, threads=4)
        conv = lambda x, w, **kw: orc.approx_conv2d_i16(bits, x, w, func=(kind, param), threads=4, **kw)
    # linear: M spans several row tiles and a ragged tail, N a ragged channel tile
    M, K, N = 300, 70, 21
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = _rand_i16(rng, (N, K), bits)
    bias = rng.standard_normal(N).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    acc = lin(orc.quantize_i16(x, s_x, bits), w)
    s_out = np.float32(s_x) * np.float32(1e-4)
    s_vec = (np.float32(s_x) * rng.uniform(1e-5, 1e-4, size=N).astype(np.float32)).astype(np.float32)
    for sc, b, act in ((s_out, None, 0), (s_out, bias, 1), (s_vec, bias, 2)):
        want = (orc.dequant_per_channel if isinstance(sc, np.ndarray) else orc.dequant)(acc, sc, M, N, 1, b)
        want = (orc.relu(want) if act == 1 else orc.tanh(want) if act == 2 else want).reshape(acc.shape)
        got = B.adapt_linear_layer_i16_f32(mul, dev(x), dev(w), s_x, dev(sc) if isinstance(sc, np.ndarray) else sc,
                                           dev(b) if b is not None else None, act)
        assert bits_equal(host(got), want), ("linear", act)
    # convolution with stride, padding and dilation
    x = rng.standard_normal((3, 5, 11, 9)).astype(np.float32)
    f = _rand_i16(rng, (7, 5, 3, 2), bits)
    bias = rng.standard_normal(7).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    acc = conv(orc.quantize_i16(x, s_x, bits), f, stride=(2, 1), pad=(1, 1), dil=(1, 2))
    n_, c_, h_, w_ = acc.shape
    s_out = np.float32(s_x) * np.float32(1e-4)
    for b, act in ((None, 0), (bias, 1), (bias, 2)):
        want = orc.dequant(acc, s_out, n_, c_, h_ * w_, b)
        want = (orc.relu(want) if act == 1 else orc.tanh(want) if act == 2 else want).reshape(acc.shape)
        got = B.adapt_conv2d_layer_i16_f32(mul, dev(x), dev(f), s_x, s_out, (2, 1), (1, 1), (1, 2), dev(b) if b is not None else None, act)
        assert bits_equal(host(got), want), ("conv", act)
    # empty batch, bad arguments
    assert B.adapt_linear_layer_i16_f32(mul, torch.zeros((0, K), device="cuda"), dev(w), 1.0, 1.0).shape == (0, N)
    with pytest.raises(B.AdaptError) as e:
        B.adapt_linear_layer_i16_f32(mul, dev(x.reshape(-1, 5)[:4]), dev(_rand_i16(rng, (3, 5), bits)), 0.0, 1.0)
    assert e.value.code == -1
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_layer_i16_f32(mul, dev(x), dev(f), 1.0, 1.0, act=3)
    assert e.value.code == -1


def test_wide_table_agrees_with_8_bit_path(B):
    """The same 8-bit table through the LDS kernels (int8 operands) and through the device-memory gather (int16)."""
    rng = np.random.default_rng(8)
    lut = wl.make_lut(8)
    a = wl.random_i8(rng, (200, 64), 8, "gauss")
    w = wl.random_i8(rng, (24, 64), 8, "gauss")
    g8 = host(B.adapt_approx_linear(B.Lut(lut, 8), dev(a), dev(w)))
    g16 = host(B.adapt_approx_linear_i16(B.Lut16(8, table=lut), dev(a.astype(np.int16)), dev(w.astype(np.int16))))
    assert (g8 == g16).all()


def test_wide_entry_points_refuse_bad_arguments(B):
    with pytest.raises(B.AdaptError) as e:
        B.Lut16(13, func=(0, 0))
    assert e.value.code == -1
    with pytest.raises(B.AdaptError) as e:
        B.adapt_approx_linear_func_i16(3, 0, 8, torch.zeros((1, 1), dtype=torch.int16, device="cuda"),
                                       torch.zeros((1, 1), dtype=torch.int16, device="cuda"))
    assert e.value.code == -1
    with pytest.raises(B.AdaptError):
        B.adapt_quantize_i16_f32(torch.zeros(4, device="cuda"), 0.0, 12)


# ------------------------------------------------------------------ the workloads beyond the baseline at the sizes bench.py times

def test_separable_block_full_size_as_benchmarked(B):
    """bench.py --config 6: depthwise 3x3 + pointwise 1x1, batch 32, 128 channels, 32x32; whole tensors."""
    from oracle import networks as onet
    from paper_2203_04071_amd import networks as gnet
    cfg = wl.separable_workload(batch=32, cin=128, cout=128, hw=32)
    want = onet.separable_conv(cfg, threads=orc.host_threads())
    net = gnet.SeparableConv(cfg)
    net.forward(dev(cfg["x"]))                  # calibration
    first = net.forward(dev(cfg["x"]), fused=False)
    assert (host(first["acc_dw"]) == want["acc_dw"]).all()
    got = gnet.Captured(net, dev(cfg["x"])).replay()          # frozen scales, as a graph replay like the benchmark
    torch.cuda.synchronize()
    assert_f32_close(host(got["out"]), want["out"])
    assert bits_equal(host(got["out"]), host(first["out"]))


def test_gru_full_size_as_benchmarked(B):
    """bench.py --config 7: GRU 512/512, batch 64, 7-bit table; the first 12 of the 100 time steps against the oracle
    (the recurrence makes every later step depend on all earlier ones, so a defect shows in the first steps)."""
    from oracle import networks as onet
    from paper_2203_04071_amd import networks as gnet
    cfg = wl.recurrent_workload("gru", seq=100, batch=64, isz=512, hsz=512, bits=7)
    want = onet.gru(cfg, threads=orc.host_threads(), steps=12)
    net = gnet.Recurrent(cfg, "gru")
    got = net.forward(dev(cfg["x"]))
    assert net.fused_step, "the benchmark shape must fit the fused kernel"
    assert got["s_x"] == want["s_x"]
    assert (host(got["acc_ih"][:12]) == want["acc_ih"]).all()
    assert bits_equal(host(got["hs"][:12]), want["hs"])


@pytest.mark.parametrize("form", ["table", "function"])
def test_12_bit_layer_full_size_as_benchmarked(B, form):
    """bench.py --config 8 / 9: the 3x3 layer of configuration 2 with 12-bit operands; whole tensor."""
    c = wl.config2()
    th = orc.host_threads()
    s_x = orc.scale_from_amax(orc.absmax(c["x"]), 12)
    s_w = orc.scale_from_amax(orc.absmax(c["w"]), 12)
    oqx, oqw = orc.quantize_i16(c["x"], s_x, 12), orc.quantize_i16(c["w"], s_w, 12)
    qx = B.adapt_quantize_i16_f32(dev(c["x"]), s_x, 12)
    qw = B.adapt_quantize_i16_f32(dev(c["w"]), s_w, 12)
    assert (host(qx) == oqx).all() and (host(qw) == oqw).all()
    if form == "table":
        lut = wl.make_lut(12)
        got = B.adapt_approx_conv2d_i16(B.Lut16(12, table=lut), qx, qw, (1, 1), (1, 1))
        want = orc.approx_conv2d_i16(12, oqx, oqw, lut=lut, pad=(1, 1), threads=th)
    else:
        got = B.adapt_approx_conv2d_func_i16(B.FUNC_MITCHELL, 0, 12, qx, qw, (1, 1), (1, 1))
        want = orc.approx_conv2d_i16(12, oqx, oqw, func=(orc.FUNC_MITCHELL, 0), pad=(1, 1), threads=th)
    assert (host(got) == want).all()


def test_stored_small_cases(B):
    """The HIP path on the inputs of tests/golden/oracle_small_cases.json (expected values written by the oracle)."""
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "oracle_small_cases.json")) as f:
        g = json.load(f)
    L = B.Lut(wl.make_lut(4), 4)
    i8 = lambda v: dev(np.array(v, dtype=np.int8))
    c = g["linear_4bit"]
    assert host(B.adapt_approx_linear(L, i8(c["A"]), i8(c["W"]))).tolist() == c["acc"]
    c = g["conv2d_4bit_pad1"]
    assert host(B.adapt_approx_conv2d(L, i8(c["x"]), i8(c["w"]), (1, 1), (1, 1))).tolist() == c["acc"]
    c = g["conv_transpose2d_4bit_s2_p1"]
    assert host(B.adapt_approx_conv_transpose2d(L, i8(c["x"]), i8(c["w"]), 2, 1)).tolist() == c["acc"]
    c = g["quantize_8bit"]
    assert host(B.adapt_quantize_f32(dev(np.array(c["x"], dtype=np.float32)), c["scale"], 8)).tolist() == c["q"]
    c = g["lstm_cell"]
    cd = dev(np.array(c["c"], dtype=np.float32))
    hd = torch.empty((2, 2), dtype=torch.float32, device="cuda")
    B.adapt_lstm_cell_f32(dev(np.array(c["acc_ih"], dtype=np.int32)), dev(np.array(c["acc_hh"], dtype=np.int32)), 1e-3, 2e-3, None, cd, hd)
    assert host(hd).view(np.uint32).tolist() == c["h_bits"] and host(cd).view(np.uint32).tolist() == c["c_bits"]
    c = g["gru_cell"]
    hd = torch.empty((2, 2), dtype=torch.float32, device="cuda")
    B.adapt_gru_cell_f32(dev(np.array(c["acc_ih"], dtype=np.int32)), dev(np.array(c["acc_hh"], dtype=np.int32)), 1e-3, 2e-3, None, None,
                         dev(np.array(c["h"], dtype=np.float32)), hd)
    assert host(hd).view(np.uint32).tolist() == c["h_bits"]
    a = dev(np.full((64, 1), 21, dtype=np.int16))
    w = dev(np.arange(-32, 32, dtype=np.int16).reshape(64, 1))
    assert host(B.adapt_approx_linear_func_i16(B.FUNC_MITCHELL, 0, 6, a, w))[0].tolist() == g["mitchell_6bit_row_of_21"]

# ------------------------------------------------------------------ random shapes through every entry point

@pytest.mark.parametrize("seed", seeds(11, 12))
def test_random_shapes_match_oracle(B, seed):
    """Seeded random shapes (ragged sizes, strides, dilations, groups, table widths incl. a two-pass table, fused layer
    calls with bias / residual / activations, transposed convolutions, function multipliers) against the oracle: exercises
    the choice between kernels at sizes nobody picked by hand."""
    ncases = 120
    rng = np.random.default_rng(seed)
    luts = {b: wl.make_lut(b) for b in (4, 6, 7, 8)}
    big = (rng.integers(-2**20, 2**20, size=(64, 64))).astype(np.int32)   # two-pass table at 6 bits
    L = {b: B.Lut(luts[b], b) for b in luts}
    Lbig = B.Lut(big, 6)
    bad = []
    for it in range(ncases):
        kind = rng.choice(["linear", "conv", "convg", "convt", "layer", "convt_layer", "lin_layer", "i16"])
        bits = int(rng.choice([4, 6, 7, 8]))
        two = bits == 6 and rng.random() < 0.3
        lut, LL = (big, Lbig) if two else (luts[bits], L[bits])
        desc = None
        try:
            if kind == "linear" or kind == "lin_layer":
                M = int(rng.choice([1, 3, 64, 130, 4096, 4100, 5000])); K = int(rng.integers(1, 200)); N = int(rng.integers(1, 70))
                a = wl.random_i8(rng, (M, K), bits, "gauss"); w = wl.random_i8(rng, (N, K), bits, "gauss")
                desc = (kind, bits, two, M, K, N)
                want = orc.approx_linear(lut, bits, a, w, threads=8)
                if kind == "linear":
                    got = host(B.adapt_approx_linear(LL, dev(a), dev(w)))
                    ok = (got == want).all()
                    pw = B.adapt_weights_pack_linear(LL, dev(w))
                    ok = ok and (host(B.adapt_approx_linear_packed(pw, dev(a))) == want).all()
                else:
                    x = (rng.standard_normal((M, K))).astype(np.float32)
                    s_x = orc.scale_from_amax(orc.absmax(x), bits)
                    qa = orc.quantize(x, s_x, bits)
                    want = orc.approx_linear(lut, bits, qa, w, threads=8)
                    bias = rng.standard_normal(N).astype(np.float32)
                    y = orc.dequant(want, np.float32(s_x) * np.float32(0.01), M, N, 1, bias)
                    y = np.maximum(y, 0)
                    pw = B.adapt_weights_pack_linear(LL, dev(w))
                    got = host(B.adapt_linear_layer_f32(pw, dev(x), s_x, np.float32(s_x) * np.float32(0.01), bias=dev(bias), act=B.ACT_RELU))
                    ok = np.array_equal(got.view(np.uint32), y.view(np.uint32))
            elif kind in ("conv", "convg", "layer"):
                g = 1
                if kind == "convg":
                    g = int(rng.choice([2, 3, 4, 8]))
                cg = int(rng.integers(1, 20)); og = int(rng.integers(1, 20))
                if kind == "convg" and rng.random() < 0.4:
                    cg, og = 1, int(rng.choice([1, 1, 2]))
                    g = int(rng.integers(2, 40))
                Cin, Cout = cg * g, og * g
                if kind != "convg" and rng.random() < 0.5:
                    Cin = int(rng.choice([8, 16, 32, 64, 96])); Cout = int(rng.choice([8, 16, 24, 64])); cg, og = Cin, Cout
                N = int(rng.choice([1, 2, 5, 16])); H = int(rng.integers(3, 40)); W = int(rng.integers(3, 40))
                kh = int(rng.choice([1, 3, 5])); kw = int(rng.choice([1, 3, 5]))
                sh = int(rng.choice([1, 1, 2])); sw = int(rng.choice([1, 1, 2])); ph = int(rng.integers(0, 3)); pw_ = int(rng.integers(0, 3))
                dh = int(rng.choice([1, 1, 2])); dw = int(rng.choice([1, 1, 2]))
                if H + 2 * ph < dh * (kh - 1) + 1 or W + 2 * pw_ < dw * (kw - 1) + 1:
                    continue
                x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss"); w = wl.random_i8(rng, (Cout, cg, kh, kw), bits, "gauss")
                desc = (kind, bits, two, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw_, dh, dw, g)
                want = orc.approx_conv2d(lut, bits, x, w, (sh, sw), (ph, pw_), (dh, dw), g, threads=8)
                if kind != "layer":
                    got = host(B.adapt_approx_conv2d(LL, dev(x), dev(w), (sh, sw), (ph, pw_), (dh, dw), groups=g))
                    ok = (got == want).all()
                    if g == 1:
                        pk = B.adapt_weights_pack_conv2d(LL, dev(w))
                        ok = ok and (host(B.adapt_approx_conv2d_packed(pk, dev(x), (sh, sw), (ph, pw_), (dh, dw))) == want).all()
                else:
                    xf = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
                    s_x = orc.scale_from_amax(orc.absmax(xf), bits)
                    qx = orc.quantize(xf, s_x, bits)
                    want = orc.approx_conv2d(lut, bits, qx, w, (sh, sw), (ph, pw_), (dh, dw), 1, threads=8)
                    n_, c_, h_, w_ = want.shape
                    bias = rng.standard_normal(Cout).astype(np.float32)
                    res = rng.standard_normal(want.shape).astype(np.float32)
                    s_o = np.float32(s_x) * np.float32(0.02)
                    y = orc.dequant(want, s_o, n_, c_, h_ * w_, bias)
                    y = np.maximum(orc.add(y, res), 0)
                    pk = B.adapt_weights_pack_conv2d(LL, dev(w))
                    got = host(B.adapt_conv2d_layer_f32(pk, dev(xf), s_x, s_o, (sh, sw), (ph, pw_), (dh, dw), bias=dev(bias), act=B.ACT_RELU, residual=dev(res)))
                    ok = np.array_equal(got.view(np.uint32), y.view(np.uint32))
            elif kind in ("convt", "convt_layer"):
                N = int(rng.choice([1, 2, 9, 40])); Cin = int(rng.integers(1, 40)); Cout = int(rng.integers(1, 30))
                H = int(rng.integers(1, 12)); W = int(rng.integers(1, 12)); k = int(rng.choice([2, 3, 4, 5])); s = int(rng.choice([1, 2, 3])); p = int(rng.integers(0, 3))
                if (H - 1) * s - 2 * p + k < 1 or (W - 1) * s - 2 * p + k < 1:
                    continue
                x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss"); w = wl.random_i8(rng, (Cin, Cout, k, k), bits, "gauss")
                desc = (kind, bits, two, N, Cin, H, W, Cout, k, s, p)
                want = orc.approx_conv_transpose2d(lut, bits, x, w, s, p, threads=8)
                pk = B.adapt_weights_pack_conv_transpose2d(LL, dev(w), s)
                if kind == "convt":
                    ok = (host(B.adapt_approx_conv_transpose2d(LL, dev(x), dev(w), s, p)) == want).all()
                    ok = ok and (host(B.adapt_approx_conv_transpose2d_packed(pk, dev(x), p)) == want).all()
                else:
                    xf = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
                    s_x = orc.scale_from_amax(orc.absmax(xf), bits)
                    want = orc.approx_conv_transpose2d(lut, bits, orc.quantize(xf, s_x, bits), w, s, p, threads=8)
                    n_, c_, h_, w_ = want.shape
                    s_o = np.float32(s_x) * np.float32(0.02)
                    act = int(rng.choice([0, 1, 2]))
                    y = orc.dequant(want, s_o, n_, c_, h_ * w_)
                    y = np.maximum(y, 0) if act == 1 else (orc.tanh(y) if act == 2 else y)
                    got = host(B.adapt_conv_transpose2d_layer_f32(pk, dev(xf), s_x, s_o, p, act=act))
                    ok = np.array_equal(got.view(np.uint32), y.view(np.uint32))
            else:
                b16 = int(rng.choice([9, 10, 12])); M = int(rng.choice([1, 70, 1030])); K = int(rng.integers(1, 60)); N = int(rng.integers(1, 20))
                h = 1 << (b16 - 1)
                a = rng.integers(-h, h, (M, K)).astype(np.int16); w = rng.integers(-h, h, (N, K)).astype(np.int16)
                kindf = int(rng.choice([0, 1, 2])); par = int(rng.integers(0, 4)) if kindf == 1 else 0
                desc = (kind, b16, M, K, N, kindf, par)
                ok = (host(B.adapt_approx_linear_func_i16(kindf, par, b16, dev(a), dev(w))) == orc.approx_linear_func_i16(kindf, par, b16, a, w, threads=8)).all()
        except B.AdaptError as e:
            bad.append((desc, str(e)))
            continue
        if not ok:
            bad.append(desc)
    assert not bad, bad


@pytest.mark.parametrize("seed", seeds(41, 42))
def test_random_long_products_match_oracle(B, seed):
    """Seeded random shapes with thousands of rows and 16 to 128 channels - what the kernels that stream derived tables
    take, unsplit or with the inner dimension in slices: convolutions (filters 1 to 5 wide, vertical stride, dilation,
    padding; as integer products and as fp32 layers), long linear products, stride-2 transposed layers with every
    activation."""
    rng = np.random.default_rng(seed)
    luts = {b: wl.make_lut(b) for b in (5, 6, 7, 8)}
    L = {b: B.Lut(luts[b], b) for b in luts}
    th = orc.host_threads()
    bad = []
    for it in range(60):
        bits = int(rng.choice([5, 6, 7, 8])); lut = luts[bits]; LL = L[bits]
        kind = str(rng.choice(["conv", "conv_layer", "linear", "convt_layer"]))
        if kind in ("conv", "conv_layer"):
            N = int(rng.choice([4, 8, 16, 32, 64, 100])); Cin = int(rng.choice([16, 32, 48, 64, 128, 20, 40]))
            Cout = int(rng.choice([5, 8, 16, 24, 32, 64, 70]))
            H = int(rng.choice([8, 10, 12, 16, 20, 32])); W = int(rng.choice([8, 12, 16, 20, 32, 36]))
            kh = int(rng.choice([1, 3, 3, 5])); kw = int(rng.choice([1, 3, 3, 5])); dh = int(rng.choice([1, 1, 2])); dw = int(rng.choice([1, 1, 2]))
            sh = int(rng.choice([1, 1, 2])); ph = int(rng.integers(0, 3))
            pw_ = (dw * (kw - 1)) // 2 if rng.random() < 0.7 else int(rng.integers(0, 3))
            if H + 2 * ph < dh * (kh - 1) + 1 or W + 2 * pw_ < dw * (kw - 1) + 1:
                continue
            w = wl.random_i8(rng, (Cout, Cin, kh, kw), bits, "gauss")
            desc = (kind, bits, N, Cin, H, W, Cout, kh, kw, sh, ph, pw_, dh, dw)
            pk = B.adapt_weights_pack_conv2d(LL, dev(w))
            if kind == "conv":
                x = wl.random_i8(rng, (N, Cin, H, W), bits, "gauss")
                want = orc.approx_conv2d(lut, bits, x, w, (sh, 1), (ph, pw_), (dh, dw), 1, threads=th)
                ok = (host(B.adapt_approx_conv2d_packed(pk, dev(x), (sh, 1), (ph, pw_), (dh, dw))) == want).all()
            else:
                xf = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
                s_x = orc.scale_from_amax(orc.absmax(xf), bits)
                want = orc.approx_conv2d(lut, bits, orc.quantize(xf, s_x, bits), w, (sh, 1), (ph, pw_), (dh, dw), 1, threads=th)
                n_, c_, h_, w_ = want.shape
                bias = rng.standard_normal(Cout).astype(np.float32); s_o = np.float32(s_x) * np.float32(0.02)
                act = int(rng.choice([0, 1]))
                y = orc.dequant(want, s_o, n_, c_, h_ * w_, bias)
                if act:
                    y = orc.relu(y)
                got = host(B.adapt_conv2d_layer_f32(pk, dev(xf), s_x, s_o, (sh, 1), (ph, pw_), (dh, dw), bias=dev(bias), act=act))
                ok = bits_equal(got, y.reshape(got.shape))
        elif kind == "linear":
            M = int(rng.choice([4096, 6400, 8192, 10000, 16384])); K = int(rng.choice([64, 96, 128, 200, 512])); N = int(rng.choice([8, 16, 30, 64]))
            a = wl.random_i8(rng, (M, K), bits, "gauss"); w = wl.random_i8(rng, (N, K), bits, "gauss")
            desc = (kind, bits, M, K, N)
            pw = B.adapt_weights_pack_linear(LL, dev(w))
            ok = (host(B.adapt_approx_linear_packed(pw, dev(a))) == orc.approx_linear(lut, bits, a, w, threads=th)).all()
        else:
            N = int(rng.choice([8, 32, 64, 128])); Cin = int(rng.choice([16, 24, 32, 64, 128])); Cout = int(rng.choice([3, 8, 16, 32, 64]))
            H = int(rng.choice([4, 8, 16])); W = int(rng.choice([4, 8, 16])); k = int(rng.choice([2, 4, 4, 6])); p = int(rng.choice([0, 1, 2]))
            if (H - 1) * 2 - 2 * p + k < 1 or (W - 1) * 2 - 2 * p + k < 1:
                continue
            w = wl.random_i8(rng, (Cin, Cout, k, k), bits, "gauss")
            xf = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
            desc = (kind, bits, N, Cin, H, W, Cout, k, p)
            s_x = orc.scale_from_amax(orc.absmax(xf), bits)
            want = orc.approx_conv_transpose2d(lut, bits, orc.quantize(xf, s_x, bits), w, 2, p, threads=th)
            n_, c_, h_, w_ = want.shape
            s_o = np.float32(s_x) * np.float32(0.02); act = int(rng.choice([0, 1, 2]))
            y = orc.dequant(want, s_o, n_, c_, h_ * w_)
            y = orc.relu(y) if act == 1 else (orc.tanh(y) if act == 2 else y)
            pk = B.adapt_weights_pack_conv_transpose2d(LL, dev(w), 2)
            got = host(B.adapt_conv_transpose2d_layer_f32(pk, dev(xf), s_x, s_o, p, act=act))
            ok = bits_equal(got, y.reshape(got.shape))
        if not ok:
            bad.append(desc)
    assert not bad, bad


@pytest.mark.parametrize("seed", seeds(21, 22))
def test_random_grouped_layers_match_oracle(B, seed):
    """Seeded random depthwise-style layers through the one-kernel layer call (fp32 in, scalar or per-channel output
    scale, bias, activation), half of them chained into a following 1x1 or 3x3 layer: y and the consumer's output
    bit-identical to the oracle's separate steps."""
    rng = np.random.default_rng(seed)
    bad, ran = [], 0
    for it in range(70):
        bits = int(rng.choice([5, 6, 8]))
        lut = wl.make_lut(bits)
        L = B.Lut(lut, bits)
        cg = int(rng.choice([1, 1, 1, 2, 3])); og = int(rng.choice([1, 1, 2, 3, 4])); g = int(rng.integers(2, 48))
        Cin, Cout = cg * g, og * g
        N = int(rng.choice([1, 2, 5])); H = int(rng.integers(3, 45)); W = int(rng.integers(3, 45))
        kh = int(rng.choice([1, 3, 5])); kw = int(rng.choice([1, 3, 3, 5]))
        sh = int(rng.choice([1, 1, 2])); sw = int(rng.choice([1, 1, 2])); ph = int(rng.integers(0, 3)); pw_ = int(rng.integers(0, 3))
        dh = int(rng.choice([1, 1, 2])); dw = int(rng.choice([1, 1, 1, 2]))
        if H + 2 * ph < dh * (kh - 1) + 1 or W + 2 * pw_ < dw * (kw - 1) + 1:
            continue
        act = int(rng.choice([0, 1, 2])); use_bias = rng.random() < 0.6; per_ch = rng.random() < 0.4
        chain = rng.random() < 0.5
        k2 = int(rng.choice([1, 3])); c2 = int(rng.choice([3, 8, 16, 64]))
        desc = (bits, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw_, dh, dw, g, act, use_bias, per_ch, chain, k2, c2)
        x = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
        w = wl.random_i8(rng, (Cout, cg, kh, kw), bits, "gauss")
        bias = rng.standard_normal(Cout).astype(np.float32) if use_bias else None
        s_x = orc.scale_from_amax(orc.absmax(x), bits)
        acc = orc.approx_conv2d(lut, bits, orc.quantize(x, s_x, bits), w, (sh, sw), (ph, pw_), (dh, dw), g, threads=8)
        n_, c_, h_, w_ = acc.shape
        if per_ch:
            sc = (np.float32(s_x) * rng.uniform(0.01, 0.03, size=Cout).astype(np.float32)).astype(np.float32)
            y = orc.dequant_per_channel(acc, sc, n_, c_, h_ * w_, bias)
        else:
            sc = np.float32(s_x) * np.float32(0.02)
            y = orc.dequant(acc, sc, n_, c_, h_ * w_, bias)
        y = (orc.relu(y) if act == 1 else orc.tanh(y) if act == 2 else y).reshape(acc.shape)
        try:
            kw_args = {}
            if chain:
                s_y = orc.scale_from_amax(orc.absmax(y), bits)
                if not s_y > 0:
                    continue
                w2 = wl.random_i8(rng, (c2, Cout, k2, k2), bits, "gauss")
                acc2 = orc.approx_conv2d(lut, bits, orc.quantize(y, s_y, bits), w2, (1, 1), (k2 // 2, k2 // 2), threads=8)
                want2 = orc.dequant(acc2, np.float32(s_y) * np.float32(0.01), n_, c2, h_ * w_).reshape(acc2.shape)
                p2 = B.adapt_weights_pack_conv2d(L, dev(w2))
                B.adapt_conv2d_chain_prepare(p2, N, h_, w_, (1, 1), (k2 // 2, k2 // 2))
                kw_args = dict(next_pw=p2, s_next=s_y)
            got = B.adapt_conv2d_grouped_layer_f32(L, dev(x), dev(w), s_x, dev(sc) if per_ch else sc, (sh, sw), (ph, pw_), (dh, dw), g,
                                                   dev(bias) if use_bias else None, act, **kw_args)
            ok = bits_equal(host(got), y)
            if chain:
                out2 = torch.empty(acc2.shape, dtype=torch.float32, device="cuda")
                B.adapt_conv2d_layer_chain_f32(p2, None, s_y, np.float32(s_y) * np.float32(0.01), out2, (1, 1), (k2 // 2, k2 // 2),
                                               in_shape=(N, h_, w_))
                ok = ok and bits_equal(host(out2), want2)
            ran += 1
        except B.AdaptError as e:
            if e.code != -2:                    # (-2: a shape the layer kernel does not take; the separate calls serve it)
                bad.append((desc, str(e)))
            continue
        if not ok:
            bad.append(desc)
    assert not bad, bad
    assert ran >= 50


# ------------------------------------------------------------------ chained convolution layers

CHAIN_CASES = [
    # N, C0, H, W, channels of three 3x3 layers, stride of the second, bits
    (32, 64, 32, 32, (64, 64, 64), 1, 8),      # quad kernel producers and consumers (as configuration 2)
    (16, 64, 8, 8, (64, 64, 64), 1, 8),        # inner dimension split over workgroups: the adding kernel writes the chain
    (8, 16, 32, 32, (16, 16, 32), 2, 8),       # paired taps, x-major; then a stride-2 consumer with a channel-last copy
    (4, 32, 16, 16, (32, 32, 32), 1, 8),       # 4 rows per lane, channel-last copies
    (3, 5, 9, 7, (7, 12, 9), 1, 6),            # ragged everything: generic kernels
    (2, 8, 12, 12, (24, 8, 16), 2, 7),
]


@pytest.mark.parametrize("case", CHAIN_CASES)
def test_chained_conv_layers_match_unchained_and_oracle(B, case):
    """Three convolution layers (bias + ReLU, residual on the last) where each layer writes the next layer's quantised,
    padded input copy in its epilogue: fp32 outputs of every layer bit-identical to the oracle's layer-by-layer pass."""
    N, C0, H, W, chans, s2, bits = case
    rng = np.random.default_rng(sum(case[:4]) + bits)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    x = rng.standard_normal((N, C0, H, W)).astype(np.float32)
    cin = C0
    ws, bs, strides = [], [], [1, s2, 1]
    for c in chans:
        ws.append(wl.random_i8(rng, (c, cin, 3, 3), bits, "gauss"))
        bs.append(rng.standard_normal(c).astype(np.float32) * np.float32(0.1))
        cin = c
    # oracle pass, layer by layer, calibrating scales progressively
    th = orc.host_threads()
    acts, scales = [x], []
    for i in range(3):
        s_x = orc.scale_from_amax(orc.absmax(acts[-1]), bits)
        scales.append(s_x)
        acc = orc.approx_conv2d(lut, bits, orc.quantize(acts[-1], s_x, bits), ws[i], (strides[i],) * 2, (1, 1), threads=th)
        n_, c_, h_, w_ = acc.shape
        y = orc.dequant(acc, np.float32(s_x) * np.float32(0.01), n_, c_, h_ * w_, bs[i])
        if i == 2 and chans[2] == chans[1]:
            y = orc.add(y, acts[-1])
        acts.append(np.maximum(y, 0))
    pws = [B.adapt_weights_pack_conv2d(L, dev(w)) for w in ws]
    shapes = [a.shape for a in acts]
    for i in (1, 2):
        B.adapt_conv2d_chain_prepare(pws[i], N, shapes[i][2], shapes[i][3], (strides[i],) * 2, (1, 1))
    outs = [torch.empty(shapes[i + 1], dtype=torch.float32, device="cuda") for i in range(3)]
    for rep in range(2):        # twice: the prepared buffers are reused
        B.adapt_conv2d_layer_chain_f32(pws[0], dev(x), scales[0], np.float32(scales[0]) * np.float32(0.01), outs[0], (1, 1), (1, 1),
                                       bias=dev(bs[0]), act=B.ACT_RELU, next_pw=pws[1], s_next=scales[1])
        B.adapt_conv2d_layer_chain_f32(pws[1], None, scales[1], np.float32(scales[1]) * np.float32(0.01), outs[1], (s2, s2), (1, 1),
                                       bias=dev(bs[1]), act=B.ACT_RELU, next_pw=pws[2], s_next=scales[2], in_shape=(N,) + shapes[1][2:])
        B.adapt_conv2d_layer_chain_f32(pws[2], None, scales[2], np.float32(scales[2]) * np.float32(0.01), outs[2], (1, 1), (1, 1),
                                       bias=dev(bs[2]), act=B.ACT_RELU, residual=outs[1] if chans[2] == chans[1] else None,
                                       in_shape=(N,) + shapes[2][2:])
        for i in range(3):
            assert bits_equal(host(outs[i]), acts[i + 1]), (rep, i)
    # the first two layers without their fp32 outputs (only the next layer's copy is wanted): the last layer's output must
    # not change; a shape that finishes its sums in a separate pass refuses (code -2) and leaves everything as it was
    outs[2].zero_()
    skipped = []
    for i, (xin, st, shp) in enumerate(((dev(x), 1, None), (None, s2, (N,) + shapes[1][2:]))):
        kw = dict(bias=dev(bs[i]), act=B.ACT_RELU, next_pw=pws[i + 1], s_next=scales[i + 1])
        if shp is not None:
            kw["in_shape"] = shp
        try:
            B.adapt_conv2d_layer_chain_f32(pws[i], xin, scales[i], np.float32(scales[i]) * np.float32(0.01), None, (st, st), (1, 1), **kw)
            skipped.append(i)
        except B.AdaptError as e:
            assert e.code == -2, e
            B.adapt_conv2d_layer_chain_f32(pws[i], xin, scales[i], np.float32(scales[i]) * np.float32(0.01), outs[i], (st, st), (1, 1), **kw)
    B.adapt_conv2d_layer_chain_f32(pws[2], None, scales[2], np.float32(scales[2]) * np.float32(0.01), outs[2], (1, 1), (1, 1),
                                   bias=dev(bs[2]), act=B.ACT_RELU, residual=outs[1] if chans[2] == chans[1] else None,
                                   in_shape=(N,) + shapes[2][2:])
    assert bits_equal(host(outs[2]), acts[3]), skipped
    if case[:4] == (32, 64, 32, 32):
        assert skipped == [0, 1]        # the layer of configuration 2 writes the copy from the product kernel
    with pytest.raises(B.AdaptError) as e:      # no output and no next layer: nothing to do
        B.adapt_conv2d_layer_chain_f32(pws[2], None, scales[2], 1.0, None, (1, 1), (1, 1), in_shape=(N,) + shapes[2][2:])
    assert e.value.code == -1


@pytest.mark.parametrize("shape", [(32, 64, 32, 32), (16, 32, 16, 16)])      # big-layer kernel; 128-byte-line kernel
@pytest.mark.parametrize("bits", [8, 7, 5])
def test_chained_consumer_after_relu_and_after_no_activation(B, bits, shape):
    """A consumer on the big-layer kernel copies only the first half of every table into LDS when the producing layer
    applied ReLU (all codes >= 0) and the whole table otherwise: the same two handles, the producer alternating between no
    activation (negative codes present) and ReLU, consumer output against the oracle every time."""
    N, C, H, W = shape
    rng = np.random.default_rng(900 + bits + N)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w0 = wl.random_i8(rng, (C, C, 3, 3), bits, "gauss")
    w1 = wl.random_i8(rng, (C, C, 3, 3), bits, "gauss")
    th = orc.host_threads()
    s0 = orc.scale_from_amax(orc.absmax(x), bits)
    acc0 = orc.approx_conv2d(lut, bits, orc.quantize(x, s0, bits), w0, (1, 1), (1, 1), threads=th)
    y0 = orc.dequant(acc0, np.float32(s0) * np.float32(0.01), N, C, H * W)
    p0, p1 = B.adapt_weights_pack_conv2d(L, dev(w0)), B.adapt_weights_pack_conv2d(L, dev(w1))
    B.adapt_conv2d_chain_prepare(p1, N, H, W, (1, 1), (1, 1))
    o0 = torch.empty((N, C, H, W), dtype=torch.float32, device="cuda")
    o1 = torch.empty((N, C, H, W), dtype=torch.float32, device="cuda")
    for act in (B.ACT_NONE, B.ACT_RELU, B.ACT_NONE, B.ACT_RELU):
        mid = np.maximum(y0, 0) if act == B.ACT_RELU else y0
        s1 = orc.scale_from_amax(orc.absmax(mid), bits)
        q1 = orc.quantize(mid, s1, bits)
        assert (q1 < 0).any() == (act == B.ACT_NONE)
        acc1 = orc.approx_conv2d(lut, bits, q1, w1, (1, 1), (1, 1), threads=th)
        want = orc.dequant(acc1, np.float32(s1) * np.float32(0.01), N, C, H * W)
        B.adapt_conv2d_layer_chain_f32(p0, dev(x), s0, np.float32(s0) * np.float32(0.01), o0, (1, 1), (1, 1), act=act, next_pw=p1, s_next=s1)
        B.adapt_conv2d_layer_chain_f32(p1, None, s1, np.float32(s1) * np.float32(0.01), o1, (1, 1), (1, 1), in_shape=(N, H, W))
        assert bits_equal(host(o0), mid), act
        assert bits_equal(host(o1), want), act


def test_refused_producer_call_does_not_change_what_the_consumer_assumes(B):
    """A producer call that is refused (no output buffer on a layer that needs one: its table takes two passes, so its
    sums are finished in a separate pass over the output) writes nothing into the next layer's copy, so it must not
    change what the consumer takes the copy to hold: the copy still has the codes of an earlier producer call WITHOUT
    ReLU (negative codes present), and the consumer has to read whole tables."""
    bits, N, C, H, W = 8, 16, 64, 16, 16
    rng = np.random.default_rng(77)
    lut = wl.make_lut(bits)
    lut_wide = rng.integers(-2**20, 2**20, size=(256, 256)).astype(np.int32)       # entries beyond 16 bits: two passes
    L, LW = B.Lut(lut, bits), B.Lut(lut_wide, bits)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w0 = wl.random_i8(rng, (C, C, 3, 3), bits, "gauss")
    w1 = wl.random_i8(rng, (C, C, 3, 3), bits, "gauss")
    th = orc.host_threads()
    s0 = orc.scale_from_amax(orc.absmax(x), bits)
    so0 = np.float32(s0) * np.float32(1e-6)
    y0 = orc.dequant(orc.approx_conv2d(lut_wide, bits, orc.quantize(x, s0, bits), w0, (1, 1), (1, 1), threads=th), so0, N, C, H * W)
    s1 = orc.scale_from_amax(orc.absmax(y0), bits)
    q1 = orc.quantize(y0, s1, bits)
    assert (q1 < 0).any()
    want = orc.dequant(orc.approx_conv2d(lut, bits, q1, w1, (1, 1), (1, 1), threads=th), np.float32(s1) * np.float32(0.01), N, C, H * W)
    p0, p1 = B.adapt_weights_pack_conv2d(LW, dev(w0)), B.adapt_weights_pack_conv2d(L, dev(w1))
    B.adapt_conv2d_chain_prepare(p1, N, H, W, (1, 1), (1, 1))
    o0 = torch.empty((N, C, H, W), dtype=torch.float32, device="cuda")
    o1 = torch.empty((N, C, H, W), dtype=torch.float32, device="cuda")
    B.adapt_conv2d_layer_chain_f32(p0, dev(x), s0, so0, o0, (1, 1), (1, 1), act=B.ACT_NONE, next_pw=p1, s_next=s1)
    assert bits_equal(host(o0), y0)
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_layer_chain_f32(p0, dev(x), s0, so0, None, (1, 1), (1, 1), act=B.ACT_RELU, next_pw=p1, s_next=s1)
    assert e.value.code == -2
    B.adapt_conv2d_layer_chain_f32(p1, None, s1, np.float32(s1) * np.float32(0.01), o1, (1, 1), (1, 1), in_shape=(N, H, W))
    assert bits_equal(host(o1), want)


GROUPED_LAYER_CASES = [
    # N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, groups, Cout of the 1x1 consumer (0: none)
    (2, 6, 5, 5, 6, 3, 3, 1, 1, 1, 1, 1, 1, 6, 0),
    (3, 32, 16, 16, 32, 3, 3, 1, 1, 1, 1, 1, 1, 32, 64),      # separable block, quad-kernel consumer
    (2, 32, 10, 10, 32, 3, 3, 1, 1, 1, 1, 1, 1, 2, 16),       # 16 output channels per group: whole-table kernel over a group dimension
    (3, 24, 9, 7, 48, 3, 3, 2, 1, 1, 0, 1, 1, 3, -8),         # 16 per group from 8, strides differ, 3x3 consumer
    (2, 5, 8, 8, 12, 3, 2, 1, 1, 1, 1, 1, 1, 1, 0),           # one group (an ordinary convolution through the same call)
    (2, 24, 15, 13, 24, 5, 5, 2, 2, 2, 2, 1, 1, 24, 10),      # 5x5 stride 2, ragged; generic consumer
    (2, 8, 9, 9, 16, 3, 3, 1, 1, 1, 1, 1, 1, 8, 12),          # channel multiplier 2
    (1, 4, 8, 8, 8, 3, 3, 1, 1, 2, 2, 2, 2, 2, 0),            # 2 groups of 2 -> 4, dilated
    (2, 12, 7, 7, 9, 3, 3, 1, 1, 1, 1, 1, 1, 3, 5),           # 3 groups of 4 -> 3
    (2, 3, 70, 70, 3, 3, 3, 1, 1, 1, 1, 1, 1, 3, 4),          # planes larger than a tile: several row chunks
    (1, 64, 8, 8, 64, 3, 3, 1, 1, 1, 1, 1, 1, 64, 32),
    (4, 128, 32, 32, 128, 3, 3, 1, 1, 1, 1, 1, 1, 128, 128),  # the benchmarked block at a smaller batch
    (8, 16, 32, 32, 16, 3, 3, 1, 1, 1, 1, 1, 1, 16, -32),     # 3x3 consumer with an x-major copy
    (3, 32, 17, 19, 32, 5, 5, 2, 2, 2, 2, 1, 1, 32, -16),     # 5x5 stride 2 into a 3x3 consumer, ragged widths
    (2, 10, 12, 12, 20, 3, 3, 1, 1, 1, 1, 1, 1, 5, 8),        # 5 groups of 2 -> 4: quads span groups
]


@pytest.mark.parametrize("bits", [6, 8])
@pytest.mark.parametrize("case", GROUPED_LAYER_CASES)
def test_grouped_conv2d_layer_f32(B, bits, case):
    """Depthwise-style layer in one kernel: quantisation of x, the sums, rescaling / bias / activation, and the quantised
    input copy of a following 1x1 layer, all against the oracle's separate steps."""
    N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, g, c_next = case
    rng = np.random.default_rng(bits + sum(case))
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    x = rng.standard_normal((N, Cin, H, W)).astype(np.float32)
    w = wl.random_i8(rng, (Cout, Cin // g, kh, kw), bits, "gauss")
    bias = rng.standard_normal(Cout).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    acc = orc.approx_conv2d(lut, bits, orc.quantize(x, s_x, bits), w, (sh, sw), (ph, pw), (dh, dw), g, threads=8)
    n_, c_, h_, w_ = acc.shape
    s_out = np.float32(s_x) * np.float32(0.02)
    s_vec = (np.float32(s_x) * rng.uniform(0.01, 0.03, size=Cout).astype(np.float32)).astype(np.float32)
    for sc, b, act in ((s_out, None, 0), (s_out, bias, 1), (s_vec, bias, 2)):
        want = (orc.dequant_per_channel if isinstance(sc, np.ndarray) else orc.dequant)(acc, sc, n_, c_, h_ * w_, b)
        want = (orc.relu(want) if act == 1 else orc.tanh(want) if act == 2 else want).reshape(acc.shape)
        got = B.adapt_conv2d_grouped_layer_f32(L, dev(x), dev(w), s_x, dev(sc) if isinstance(sc, np.ndarray) else sc, (sh, sw), (ph, pw),
                                               (dh, dw), g, dev(b) if b is not None else None, act)
        assert bits_equal(host(got), want), (b is not None, act)
    if not c_next:
        return
    # chained into a 1x1 layer: with and without the fp32 output of the grouped layer
    y = orc.relu(orc.dequant(acc, s_out, n_, c_, h_ * w_, bias)).reshape(acc.shape)
    s_y = orc.scale_from_amax(orc.absmax(y), bits)
    k2, c_next = (3, -c_next) if c_next < 0 else (1, c_next)      # negative: the consumer is a 3x3 layer with padding 1
    w2 = wl.random_i8(rng, (c_next, Cout, k2, k2), bits, "gauss")
    acc2 = orc.approx_conv2d(lut, bits, orc.quantize(y, s_y, bits), w2, (1, 1), (k2 // 2, k2 // 2), threads=8)
    want2 = orc.dequant(acc2, np.float32(s_y) * np.float32(0.01), n_, c_next, h_ * w_).reshape(acc2.shape)
    p2 = B.adapt_weights_pack_conv2d(L, dev(w2))
    B.adapt_conv2d_chain_prepare(p2, N, h_, w_, (1, 1), (k2 // 2, k2 // 2))
    out2 = torch.empty(acc2.shape, dtype=torch.float32, device="cuda")
    for want_out in ((True, True) if Cout // g >= 8 or g == 1 else (True, False, True)):     # (groups of >= 8 channels finish in place: y is needed)
        got = B.adapt_conv2d_grouped_layer_f32(L, dev(x), dev(w), s_x, s_out, (sh, sw), (ph, pw), (dh, dw), g, dev(bias), B.ACT_RELU,
                                               want_out=want_out, next_pw=p2, s_next=s_y)
        assert (got is None) == (not want_out)
        if want_out:
            assert bits_equal(host(got), y)
        out2.zero_()
        B.adapt_conv2d_layer_chain_f32(p2, None, s_y, np.float32(s_y) * np.float32(0.01), out2, (1, 1), (k2 // 2, k2 // 2),
                                       in_shape=(N, h_, w_))
        assert bits_equal(host(out2), want2), want_out


def test_grouped_layer_refusals(B):
    L = B.Lut(wl.make_lut(8), 8)
    rng = np.random.default_rng(4)
    x = torch.zeros((1, 8, 6, 1000), device="cuda")
    # input region of one output row too large to stage; groups of >= 8 channels without an output buffer; two-pass table
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_grouped_layer_f32(L, x, dev(wl.random_i8(rng, (4, 4, 5, 5), 8)), 1.0, 1.0, (1, 1), (2, 2), groups=2)
    assert e.value.code == -2
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_grouped_layer_f32(L, x, dev(wl.random_i8(rng, (16, 4, 3, 3), 8)), 1.0, 1.0, (1, 1), (1, 1), groups=2, want_out=False)
    assert e.value.code == -1
    wide = B.Lut(rng.integers(-2**20, 2**20, size=(64, 64)).astype(np.int32), 6)
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_grouped_layer_f32(wide, torch.zeros((1, 8, 6, 6), device="cuda"), dev(wl.random_i8(rng, (8, 1, 3, 3), 6)), 1.0, 1.0,
                                         (1, 1), (1, 1), groups=8)
    assert e.value.code == -2
    # a consumer that was not prepared, or prepared for another shape
    p1 = B.adapt_weights_pack_conv2d(L, dev(wl.random_i8(rng, (8, 8, 1, 1), 8)))
    xs = torch.zeros((1, 8, 6, 6), device="cuda")
    wd = dev(wl.random_i8(rng, (8, 1, 3, 3), 8))
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_grouped_layer_f32(L, xs, wd, 1.0, 1.0, (1, 1), (1, 1), groups=8, next_pw=p1, s_next=1.0)
    assert e.value.code == -1
    B.adapt_conv2d_chain_prepare(p1, 1, 5, 6)
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_grouped_layer_f32(L, xs, wd, 1.0, 1.0, (1, 1), (1, 1), groups=8, next_pw=p1, s_next=1.0)
    assert e.value.code == -1


@pytest.mark.parametrize("lo,span", [(-32768, 32895), (-16384, 32895), (-128, 32895), (-20000, 32896), (-3, 7), (-32768, 65535)])
def test_quad_kernel_table_ranges(B, lo, span):
    """The big-layer kernel stores every table entry as two int8 digits of (entry - offset), offset = smallest entry +
    32640, which covers any 16-bit range: tables whose entries sit at both ends of a range, ranges around the limit of the
    kernel's predecessor (32895), tiny and full int16 ranges, on a layer shape that takes that kernel; sums bit-exact."""
    bits = 8
    rng = np.random.default_rng(abs(lo) + span)
    hi = lo + span
    lut = rng.integers(lo, hi + 1, size=(256, 256), dtype=np.int64)
    lut[0, 0], lut[255, 255], lut[128, 128], lut[7, 200] = lo, hi, hi, lo      # both extremes present, also for operand 0
    lut = lut.astype(np.int32)
    L = B.Lut(lut, bits)
    N, Cin, Cout, HW = 32, 32, 64, 32
    x = wl.random_i8(rng, (N, Cin, HW, HW), bits, "gauss")
    w = wl.random_i8(rng, (Cout, Cin, 3, 3), bits, "gauss")
    want = orc.approx_conv2d(lut, bits, x, w, (1, 1), (1, 1), threads=orc.host_threads())
    pw = B.adapt_weights_pack_conv2d(L, dev(w))
    got = host(B.adapt_approx_conv2d_packed(pw, dev(x), (1, 1), (1, 1)))
    assert (got == want).all()
    # the same through the fused layer call (rescaling in the kernel's epilogue)
    xf = rng.standard_normal((N, Cin, HW, HW)).astype(np.float32)
    s_x = orc.scale_from_amax(orc.absmax(xf), bits)
    acc = orc.approx_conv2d(lut, bits, orc.quantize(xf, s_x, bits), w, (1, 1), (1, 1), threads=orc.host_threads())
    y = orc.dequant(acc, np.float32(1e-6), N, Cout, HW * HW).reshape(acc.shape)
    assert bits_equal(host(B.adapt_conv2d_layer_f32(pw, dev(xf), s_x, np.float32(1e-6), (1, 1), (1, 1))), y)


@pytest.mark.parametrize("seed", seeds(31, 32))
def test_random_chains_match_oracle(B, seed):
    """Seeded random pairs of convolution layers, the first writing the second's quantised input copy in its epilogue:
    channel counts, image sizes, filter sizes, strides, paddings and table widths nobody picked by hand, so that every
    producer kernel (quad, paired taps, generic, split sums) meets every copy layout."""
    rng = np.random.default_rng(seed)
    bad, ran = [], 0
    th = orc.host_threads()
    for it in range(40):
        bits = int(rng.choice([5, 6, 7, 8]))
        lut = wl.make_lut(bits)
        L = B.Lut(lut, bits)
        N = int(rng.choice([1, 2, 5, 16, 33]))
        C0 = int(rng.choice([3, 8, 16, 24, 32, 64])); C1 = int(rng.choice([4, 8, 16, 32, 40, 64])); C2 = int(rng.choice([3, 8, 16, 32, 64]))
        H = int(rng.integers(4, 34)); W = int(rng.integers(4, 34))
        k1 = int(rng.choice([1, 3, 3])); s1 = int(rng.choice([1, 1, 2])); p1 = int(rng.integers(0, k1 // 2 + 1))
        k2 = int(rng.choice([1, 3, 3, 5])); s2 = int(rng.choice([1, 1, 2])); p2 = int(rng.integers(0, k2 // 2 + 2))
        d2 = int(rng.choice([1, 1, 2]))
        H1 = (H + 2 * p1 - k1) // s1 + 1; W1 = (W + 2 * p1 - k1) // s1 + 1
        if H1 < 1 or W1 < 1 or H1 + 2 * p2 < d2 * (k2 - 1) + 1 or W1 + 2 * p2 < d2 * (k2 - 1) + 1:
            continue
        act = int(rng.choice([0, 1])); use_res = rng.random() < 0.3
        desc = (bits, N, C0, H, W, C1, k1, s1, p1, C2, k2, s2, p2, d2, act, use_res)
        x = rng.standard_normal((N, C0, H, W)).astype(np.float32)
        w1 = wl.random_i8(rng, (C1, C0, k1, k1), bits, "gauss"); w2 = wl.random_i8(rng, (C2, C1, k2, k2), bits, "gauss")
        b1 = rng.standard_normal(C1).astype(np.float32) * np.float32(0.1)
        s_x = orc.scale_from_amax(orc.absmax(x), bits)
        acc1 = orc.approx_conv2d(lut, bits, orc.quantize(x, s_x, bits), w1, (s1, s1), (p1, p1), threads=th)
        y1 = orc.dequant(acc1, np.float32(s_x) * np.float32(0.02), N, C1, H1 * W1, b1)
        res = rng.standard_normal(acc1.shape).astype(np.float32) if use_res else None
        if use_res:
            y1 = orc.add(y1, res)
        y1 = (orc.relu(y1) if act == 1 else y1).reshape(acc1.shape)
        s_y = orc.scale_from_amax(orc.absmax(y1), bits)
        if not s_y > 0:
            continue
        acc2 = orc.approx_conv2d(lut, bits, orc.quantize(y1, s_y, bits), w2, (s2, s2), (p2, p2), (d2, d2), threads=th)
        y2 = orc.dequant(acc2, np.float32(s_y) * np.float32(0.01), N, C2, acc2.shape[2] * acc2.shape[3]).reshape(acc2.shape)
        try:
            pa = B.adapt_weights_pack_conv2d(L, dev(w1)); pb = B.adapt_weights_pack_conv2d(L, dev(w2))
            B.adapt_conv2d_chain_prepare(pb, N, H1, W1, (s2, s2), (p2, p2), (d2, d2))
            o1 = torch.empty(acc1.shape, dtype=torch.float32, device="cuda")
            o2 = torch.empty(acc2.shape, dtype=torch.float32, device="cuda")
            ok = True
            for rep in range(2):
                B.adapt_conv2d_layer_chain_f32(pa, dev(x), s_x, np.float32(s_x) * np.float32(0.02), o1, (s1, s1), (p1, p1), bias=dev(b1),
                                               act=act, residual=dev(res) if use_res else None, next_pw=pb, s_next=s_y)
                o2.zero_()
                B.adapt_conv2d_layer_chain_f32(pb, None, s_y, np.float32(s_y) * np.float32(0.01), o2, (s2, s2), (p2, p2), (d2, d2),
                                               in_shape=(N, H1, W1))
                ok = ok and bits_equal(host(o1), y1) and bits_equal(host(o2), y2)
            ran += 1
        except B.AdaptError as e:
            bad.append((desc, str(e)))
            continue
        if not ok:
            bad.append(desc)
    assert not bad, bad
    assert ran >= 25


CONVT_CHAIN_CASES = [
    # N, C0, H, W, (C1, k1, s1, p1), consumer ("t" transposed / "c" ordinary, C2, k2, s2, p2), bits
    (16, 64, 8, 8, (32, 4, 2, 1), ("t", 16, 4, 2, 1), 8),      # quad kernels on both sides, borders taken off in the epilogue
    (256, 100, 1, 1, (32, 4, 1, 0), ("t", 16, 4, 2, 1), 6),    # single input pixel (a linear layer) into a phase-form layer
    (4, 8, 5, 6, (12, 3, 2, 0), ("t", 5, 4, 2, 1), 8),         # producer in gather form (3 is no multiple of 2), ragged sizes
    (3, 7, 5, 5, (9, 2, 2, 0), ("t", 4, 2, 2, 0), 7),          # no border terms at all, generic kernels
    (8, 32, 8, 8, (32, 4, 2, 1), ("c", 16, 3, 1, 1), 8),       # into an ordinary convolution
    (32, 128, 16, 16, (64, 4, 2, 1), ("t", 8, 4, 2, 1), 8),    # long layers: several rounds of workgroups
]


@pytest.mark.parametrize("case", CONVT_CHAIN_CASES)
def test_chained_transposed_convolutions(B, case):
    """A transposed-convolution layer (ReLU) that writes the next layer's quantised input copy, the next layer run from
    that copy: both outputs bit-identical to the oracle's layer-by-layer pass; twice, to reuse the prepared buffer."""
    N, C0, H, W, (C1, k1, s1, p1), (kind2, C2, k2, s2, p2), bits = case
    rng = np.random.default_rng(sum(case[:4]) + bits + C1 + C2)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    th = orc.host_threads()
    x = rng.standard_normal((N, C0, H, W)).astype(np.float32)
    w1 = wl.random_i8(rng, (C0, C1, k1, k1), bits, "gauss")
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    acc1 = orc.approx_conv_transpose2d(lut, bits, orc.quantize(x, s_x, bits), w1, s1, p1, threads=th)
    n_, c_, h1, w1_ = acc1.shape
    y1 = orc.relu(orc.dequant(acc1, np.float32(s_x) * np.float32(0.02), n_, c_, h1 * w1_)).reshape(acc1.shape)
    s_y = orc.scale_from_amax(orc.absmax(y1), bits)
    qy = orc.quantize(y1, s_y, bits)
    if kind2 == "t":
        w2 = wl.random_i8(rng, (C1, C2, k2, k2), bits, "gauss")
        acc2 = orc.approx_conv_transpose2d(lut, bits, qy, w2, s2, p2, threads=th)
    else:
        w2 = wl.random_i8(rng, (C2, C1, k2, k2), bits, "gauss")
        acc2 = orc.approx_conv2d(lut, bits, qy, w2, (s2, s2), (p2, p2), threads=th)
    y2 = orc.tanh(orc.dequant(acc2, np.float32(s_y) * np.float32(0.01), n_, C2, acc2.shape[2] * acc2.shape[3])).reshape(acc2.shape)
    pa = B.adapt_weights_pack_conv_transpose2d(L, dev(w1), s1)
    if kind2 == "t":
        pb = B.adapt_weights_pack_conv_transpose2d(L, dev(w2), s2)
        B.adapt_conv_transpose2d_chain_prepare(pb, N, h1, w1_, p2)
    else:
        pb = B.adapt_weights_pack_conv2d(L, dev(w2))
        B.adapt_conv2d_chain_prepare(pb, N, h1, w1_, (s2, s2), (p2, p2))
    o1 = torch.empty(acc1.shape, dtype=torch.float32, device="cuda")
    o2 = torch.empty(acc2.shape, dtype=torch.float32, device="cuda")
    for rep in range(2):
        B.adapt_conv_transpose2d_layer_chain_f32(pa, dev(x), s_x, np.float32(s_x) * np.float32(0.02), o1, p1, act=B.ACT_RELU, next_pw=pb, s_next=s_y)
        o2.zero_()
        if kind2 == "t":
            B.adapt_conv_transpose2d_layer_chain_f32(pb, None, s_y, np.float32(s_y) * np.float32(0.01), o2, p2, act=B.ACT_TANH, in_shape=(N, h1, w1_))
        else:
            B.adapt_conv2d_layer_chain_f32(pb, None, s_y, np.float32(s_y) * np.float32(0.01), o2, (s2, s2), (p2, p2), act=B.ACT_TANH,
                                           in_shape=(N, h1, w1_))
        assert bits_equal(host(o1), y1), rep
        assert bits_equal(host(o2), y2), rep


def test_chain_prepare_clears_copies_beyond_4_mib(B):
    """The consumer's padded input copy (here 4.7 MB) is cleared as a whole when the chain is prepared, whatever the
    handle's workspace held before: the same handle first runs an unpadded layer whose copy fills those bytes."""
    bits, N, C0, C1, C2, HW = 6, 64, 8, 64, 16, 32
    rng = np.random.default_rng(77)
    lut = wl.make_lut(bits)
    L = B.Lut(lut, bits)
    th = orc.host_threads()
    x = rng.standard_normal((N, C0, HW, HW)).astype(np.float32)
    w1 = wl.random_i8(rng, (C1, C0, 3, 3), bits, "gauss"); w2 = wl.random_i8(rng, (C2, C1, 3, 3), bits, "gauss")
    s_x = orc.scale_from_amax(orc.absmax(x), bits)
    acc1 = orc.approx_conv2d(lut, bits, orc.quantize(x, s_x, bits), w1, (1, 1), (1, 1), threads=th)
    y1 = orc.relu(orc.dequant(acc1, np.float32(s_x) * np.float32(0.02), N, C1, HW * HW)).reshape(acc1.shape)
    s_y = orc.scale_from_amax(orc.absmax(y1), bits)
    acc2 = orc.approx_conv2d(lut, bits, orc.quantize(y1, s_y, bits), w2, (1, 1), (1, 1), threads=th)
    y2 = orc.dequant(acc2, np.float32(s_y) * np.float32(0.01), N, C2, HW * HW).reshape(acc2.shape)
    pa = B.adapt_weights_pack_conv2d(L, dev(w1)); pb = B.adapt_weights_pack_conv2d(L, dev(w2))
    junk = dev((rng.standard_normal((N, C1, HW + 2, HW + 2)) + 3).astype(np.float32))         # no zero codes anywhere
    B.adapt_conv2d_layer_f32(pb, junk, 0.1, 1.0, (1, 1), (0, 0))
    B.adapt_conv2d_chain_prepare(pb, N, HW, HW, (1, 1), (1, 1), (1, 1))
    o1 = torch.empty(acc1.shape, dtype=torch.float32, device="cuda"); o2 = torch.empty(acc2.shape, dtype=torch.float32, device="cuda")
    B.adapt_conv2d_layer_chain_f32(pa, dev(x), s_x, np.float32(s_x) * np.float32(0.02), o1, (1, 1), (1, 1), act=B.ACT_RELU, next_pw=pb, s_next=s_y)
    B.adapt_conv2d_layer_chain_f32(pb, None, s_y, np.float32(s_y) * np.float32(0.01), o2, (1, 1), (1, 1), (1, 1), in_shape=(N, HW, HW))
    assert bits_equal(host(o1), y1)
    assert bits_equal(host(o2), y2)


def test_transposed_chain_refusals(B):
    L = B.Lut(wl.make_lut(8), 8)
    rng = np.random.default_rng(6)
    p3 = B.adapt_weights_pack_conv_transpose2d(L, dev(wl.random_i8(rng, (8, 8, 3, 3), 8)), 2)      # 3 is no multiple of 2: no phase form
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv_transpose2d_chain_prepare(p3, 2, 5, 5, 0)
    assert e.value.code == -2
    p4 = B.adapt_weights_pack_conv_transpose2d(L, dev(wl.random_i8(rng, (8, 8, 4, 4), 8)), 2)
    y = torch.empty((2, 8, 10, 10), device="cuda")
    with pytest.raises(B.AdaptError) as e:      # not prepared
        B.adapt_conv_transpose2d_layer_chain_f32(p4, None, 1.0, 1.0, y, 1, in_shape=(2, 5, 5))
    assert e.value.code == -1
    B.adapt_conv_transpose2d_chain_prepare(p4, 2, 5, 5, 1)
    with pytest.raises(B.AdaptError) as e:      # prepared for another size
        B.adapt_conv_transpose2d_layer_chain_f32(p4, None, 1.0, 1.0, y, 1, in_shape=(2, 6, 5))
    assert e.value.code == -1
    pa = B.adapt_weights_pack_conv_transpose2d(L, dev(wl.random_i8(rng, (8, 8, 4, 4), 8)), 2)
    x = torch.zeros((2, 8, 3, 3), device="cuda")
    y6 = torch.empty((2, 8, 6, 6), device="cuda")
    with pytest.raises(B.AdaptError) as e:      # the consumer expects 5 x 5 inputs, this layer makes 6 x 6
        B.adapt_conv_transpose2d_layer_chain_f32(pa, x, 1.0, 1.0, y6, 1, next_pw=p4, s_next=1.0)
    assert e.value.code == -1


def test_chain_refuses_unprepared_handles(B):
    L = B.Lut(wl.make_lut(8), 8)
    rng = np.random.default_rng(3)
    p0 = B.adapt_weights_pack_conv2d(L, dev(wl.random_i8(rng, (8, 8, 3, 3), 8)))
    p1 = B.adapt_weights_pack_conv2d(L, dev(wl.random_i8(rng, (8, 8, 3, 3), 8)))
    x = torch.zeros((1, 8, 6, 6), device="cuda")
    y = torch.empty((1, 8, 6, 6), device="cuda")
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_layer_chain_f32(p0, x, 1.0, 1.0, y, (1, 1), (1, 1), next_pw=p1, s_next=1.0)
    assert e.value.code == -1
    with pytest.raises(B.AdaptError) as e:
        B.adapt_conv2d_layer_chain_f32(p1, None, 1.0, 1.0, y, (1, 1), (1, 1), in_shape=(1, 6, 6))
    assert e.value.code == -1
    B.adapt_conv2d_chain_prepare(p1, 1, 6, 6, (1, 1), (1, 1))
    B.adapt_conv2d_layer_f32(p1, torch.zeros((2, 8, 5, 5), device="cuda"), 1.0, 1.0, (1, 1), (1, 1))      # another geometry
    with pytest.raises(B.AdaptError):
        B.adapt_conv2d_layer_chain_f32(p1, None, 1.0, 1.0, y, (1, 1), (1, 1), in_shape=(1, 6, 6))

