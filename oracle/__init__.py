"""CPU oracle for the approximate-multiplier hot path (AdaPT, arXiv 2203.04071).

TEST INFRASTRUCTURE ONLY: imported by the test-suite, the smoke check and the
benchmark's cpu_baseline leg.  The product path never imports this package, and
this package never imports the product path.

`oracle.c` holds the plain definitions (loops + table reads); this file is the
ctypes marshalling around it and `networks.py` strings the layers of the
benchmark networks together.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (-O2, no FMA contraction, OpenMP for the batch loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_absmax_f32.restype = ctypes.c_float
        _lib.orc_scale_from_amax.restype = ctypes.c_float
        _lib.orc_scale_from_amax.argtypes = [ctypes.c_float, ctypes.c_int]
        for name in ("orc_exp_f32", "orc_sigmoid_f32", "orc_tanh_f32"):
            f = getattr(_lib, name)
            f.restype = ctypes.c_float
            f.argtypes = [ctypes.c_float]
    return _lib


def host_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int8, a.dtype
    return a


def _f32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def _lut(t, bits):
    t = np.ascontiguousarray(t)
    assert t.dtype == np.int32 and t.size == (1 << bits) ** 2, (t.dtype, t.shape, bits)
    return t


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


L = ctypes.c_long


def approx_linear(lut, bits, A, W, threads: int = 1) -> np.ndarray:
    lut, A, W = _lut(lut, bits), _i8(A), _i8(W)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    _check(lib().orc_approx_linear(_p(lut), bits, _p(A), _p(W), _p(acc), L(M), L(K), L(N), int(threads)),
           "approx_linear")
    return acc


def conv_out_hw(H, W, kh, kw, sh, sw, ph, pw, dh=1, dw=1):
    return ((H + 2 * ph - dh * (kh - 1) - 1) // sh + 1, (W + 2 * pw - dw * (kw - 1) - 1) // sw + 1)


def approx_conv2d(lut, bits, x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1, threads: int = 1,
                  form: str = "direct") -> np.ndarray:
    lut, x, w = _lut(lut, bits), _i8(x), _i8(w)
    N, Cin, H, W = x.shape
    Cout, cg, kh, kw = w.shape
    assert cg * groups == Cin
    Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    acc = np.empty((N, Cout, Ho, Wo), dtype=np.int32)
    fn = lib().orc_approx_conv2d_direct if form == "direct" else lib().orc_approx_conv2d_im2col
    _check(fn(_p(lut), bits, _p(x), _p(w), _p(acc), L(N), L(Cin), L(H), L(W), L(Cout), L(kh), L(kw),
              L(stride[0]), L(stride[1]), L(pad[0]), L(pad[1]), L(dil[0]), L(dil[1]), L(groups),
              int(threads)), "approx_conv2d")
    return acc


def im2col(x, kh, kw, stride=(1, 1), pad=(0, 0), dil=(1, 1)) -> np.ndarray:
    x = _i8(x)
    N, Cin, H, W = x.shape
    Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    col = np.empty((N * Ho * Wo, Cin * kh * kw), dtype=np.int8)
    _check(lib().orc_im2col_i8(_p(x), _p(col), L(N), L(Cin), L(H), L(W), L(0), L(Cin), L(kh), L(kw),
                               L(stride[0]), L(stride[1]), L(pad[0]), L(pad[1]), L(dil[0]), L(dil[1])),
           "im2col")
    return col


def approx_conv_transpose2d(lut, bits, x, w, stride=1, pad=0, threads: int = 1) -> np.ndarray:
    lut, x, w = _lut(lut, bits), _i8(x), _i8(w)
    N, Cin, H, W = x.shape
    Cin2, Cout, kh, kw = w.shape
    assert Cin == Cin2
    Ho, Wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
    acc = np.empty((N, Cout, Ho, Wo), dtype=np.int32)
    _check(lib().orc_approx_conv_transpose2d(_p(lut), bits, _p(x), _p(w), _p(acc), L(N), L(Cin), L(H), L(W),
                                             L(Cout), L(kh), L(kw), L(stride), L(pad), int(threads)),
           "approx_conv_transpose2d")
    return acc


def absmax(x) -> np.float32:
    x = _f32(x)
    return np.float32(lib().orc_absmax_f32(_p(x), ctypes.c_size_t(x.size)))


def scale_from_amax(amax, bits) -> np.float32:
    return np.float32(lib().orc_scale_from_amax(ctypes.c_float(float(amax)), int(bits)))


def quantize(x, scale, bits) -> np.ndarray:
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.int8)
    _check(lib().orc_quantize_f32(_p(x), _p(q), ctypes.c_size_t(x.size), ctypes.c_float(float(scale)),
                                  int(bits)), "quantize")
    return q


def dequant(acc, scale, outer, channels, inner, bias=None) -> np.ndarray:
    acc = np.ascontiguousarray(acc)
    assert acc.dtype == np.int32 and acc.size == outer * channels * inner
    y = np.empty(acc.shape, dtype=np.float32)
    b = _f32(bias) if bias is not None else None
    _check(lib().orc_dequant_i32(_p(acc), _p(y), ctypes.c_size_t(outer), ctypes.c_size_t(channels),
                                 ctypes.c_size_t(inner), ctypes.c_float(float(scale)),
                                 _p(b) if b is not None else None), "dequant")
    return y


def absmax_rows(x) -> np.ndarray:
    x = _f32(x)
    rows = x.shape[0]
    cols = x.size // rows if rows else 0
    out = np.empty(rows, dtype=np.float32)
    _check(lib().orc_absmax_rows_f32(_p(x), ctypes.c_size_t(rows), ctypes.c_size_t(cols), _p(out)), "absmax_rows")
    return out


def quantize_rows(x, scales, bits) -> np.ndarray:
    x = _f32(x)
    scales = _f32(scales)
    rows = x.shape[0]
    cols = x.size // rows
    q = np.empty(x.shape, dtype=np.int8)
    _check(lib().orc_quantize_rows_f32(_p(x), _p(q), ctypes.c_size_t(rows), ctypes.c_size_t(cols), _p(scales), int(bits)),
           "quantize_rows")
    return q


def dequant_per_channel(acc, scales, outer, channels, inner, bias=None) -> np.ndarray:
    acc = np.ascontiguousarray(acc)
    scales = _f32(scales)
    assert acc.dtype == np.int32 and acc.size == outer * channels * inner and scales.size == channels
    y = np.empty(acc.shape, dtype=np.float32)
    b = _f32(bias) if bias is not None else None
    _check(lib().orc_dequant_i32_per_channel(_p(acc), _p(y), ctypes.c_size_t(outer), ctypes.c_size_t(channels),
                                             ctypes.c_size_t(inner), _p(scales), _p(b) if b is not None else None),
           "dequant_per_channel")
    return y


def histogram_abs(x, amax, bins, counts=None) -> np.ndarray:
    x = _f32(x)
    if counts is None:
        counts = np.zeros(bins, dtype=np.uint32)
    assert counts.dtype == np.uint32 and counts.size == bins
    _check(lib().orc_histogram_abs_f32(_p(x), ctypes.c_size_t(x.size), ctypes.c_float(float(amax)), int(bins), _p(counts)),
           "histogram_abs")
    return counts


def percentile_from_histogram(counts, amax, num=999, den=1000) -> np.float32:
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    out = ctypes.c_float(0.0)
    _check(lib().orc_percentile_from_histogram(_p(counts), int(counts.size), ctypes.c_float(float(amax)),
                                               ctypes.c_ulonglong(num), ctypes.c_ulonglong(den), ctypes.byref(out)),
           "percentile_from_histogram")
    return np.float32(out.value)


def mse_from_histogram(counts, amax, bits) -> np.float32:
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    out = ctypes.c_float(0.0)
    _check(lib().orc_mse_from_histogram(_p(counts), int(counts.size), ctypes.c_float(float(amax)), ctypes.c_int(bits),
                                        ctypes.byref(out)), "mse_from_histogram")
    return np.float32(out.value)


def entropy_from_histogram(counts, amax, bits, with_losses=False):
    """calib_max by smallest Kullback-Leibler loss (see orc_entropy_from_histogram); with_losses: also KL_k, k = 1 .. bins."""
    counts = np.ascontiguousarray(counts, dtype=np.uint32)
    out = ctypes.c_float(0.0)
    kl = np.empty(counts.size, dtype=np.float64) if with_losses else None
    _check(lib().orc_entropy_from_histogram(_p(counts), int(counts.size), ctypes.c_float(float(amax)), ctypes.c_int(bits),
                                            ctypes.byref(out), _p(kl) if with_losses else None), "entropy_from_histogram")
    return (np.float32(out.value), kl) if with_losses else np.float32(out.value)


def relu(x) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().orc_relu_f32(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def add(a, b) -> np.ndarray:
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().orc_add_f32(_p(a), _p(b), _p(y), ctypes.c_size_t(a.size))
    return y


def avgpool_hw(x) -> np.ndarray:
    x = _f32(x)
    N, C, H, W = x.shape
    y = np.empty((N, C), dtype=np.float32)
    lib().orc_avgpool_hw_f32(_p(x), _p(y), ctypes.c_size_t(N * C), ctypes.c_size_t(H * W))
    return y


def shortcut_a(x, cout) -> np.ndarray:
    x = _f32(x)
    N, C, H, W = x.shape
    y = np.empty((N, cout, (H + 1) // 2, (W + 1) // 2), dtype=np.float32)
    lib().orc_shortcut_a_f32(_p(x), _p(y), L(N), L(C), L(H), L(W), L(cout))
    return y


def _vec(fn, x):
    x = _f32(x)
    y = np.empty_like(x)
    fn(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def tanh(x):
    return _vec(lib().orc_tanh_vec_f32, x)


def sigmoid(x):
    return _vec(lib().orc_sigmoid_vec_f32, x)


def exp(x):
    return _vec(lib().orc_exp_vec_f32, x)


def lstm_cell(acc_ih, acc_hh, s_ih, s_hh, bias, c):
    """Returns (h_new, c_new); `c` is not modified."""
    acc_ih = np.ascontiguousarray(acc_ih)
    acc_hh = np.ascontiguousarray(acc_hh)
    assert acc_ih.dtype == np.int32 and acc_hh.dtype == np.int32 and acc_ih.shape == acc_hh.shape
    B, H4 = acc_ih.shape
    Hs = H4 // 4
    c2 = np.array(_f32(c), copy=True)
    h = np.empty((B, Hs), dtype=np.float32)
    b = _f32(bias) if bias is not None else None
    lib().orc_lstm_cell_f32(_p(acc_ih), _p(acc_hh), ctypes.c_float(float(s_ih)), ctypes.c_float(float(s_hh)),
                            _p(b) if b is not None else None, _p(c2), _p(h), L(B), L(Hs))
    return h, c2


def gru_cell(acc_ih, acc_hh, s_ih, s_hh, b_ih, b_hh, h):
    """Returns h_new [B][Hs]; gate order r, z, n along the 3*Hs axis."""
    acc_ih = np.ascontiguousarray(acc_ih)
    acc_hh = np.ascontiguousarray(acc_hh)
    assert acc_ih.dtype == np.int32 and acc_hh.dtype == np.int32 and acc_ih.shape == acc_hh.shape
    B, H3 = acc_ih.shape
    Hs = H3 // 3
    hp = _f32(h)
    assert hp.shape == (B, Hs)
    out = np.empty((B, Hs), dtype=np.float32)
    bi = _f32(b_ih) if b_ih is not None else None
    bh = _f32(b_hh) if b_hh is not None else None
    lib().orc_gru_cell_f32(_p(acc_ih), _p(acc_hh), ctypes.c_float(float(s_ih)), ctypes.c_float(float(s_hh)),
                           _p(bi) if bi is not None else None, _p(bh) if bh is not None else None, _p(hp), _p(out),
                           L(B), L(Hs))
    return out


def rnn_cell(acc_ih, acc_hh, s_ih, s_hh, bias, relu=False):
    """Returns h_new [B][Hs] = tanh (or ReLU) of the rescaled sums + bias."""
    acc_ih = np.ascontiguousarray(acc_ih)
    acc_hh = np.ascontiguousarray(acc_hh)
    assert acc_ih.dtype == np.int32 and acc_hh.dtype == np.int32 and acc_ih.shape == acc_hh.shape
    B, Hs = acc_ih.shape
    out = np.empty((B, Hs), dtype=np.float32)
    b = _f32(bias) if bias is not None else None
    lib().orc_rnn_cell_f32(_p(acc_ih), _p(acc_hh), ctypes.c_float(float(s_ih)), ctypes.c_float(float(s_hh)),
                           _p(b) if b is not None else None, ctypes.c_int(1 if relu else 0), _p(out), L(B), L(Hs))
    return out


# ---- operands wider than 8 bits, multipliers as functions (Sec. III-C; 12-bit unit of Sec. V)

FUNC_EXACT, FUNC_TRUNC, FUNC_MITCHELL = 0, 1, 2


def _i16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int16
    return a


def mul_func(kind, param, a, w) -> int:
    f = lib().orc_mul_func
    f.restype = ctypes.c_int32
    return int(f(ctypes.c_int(kind), ctypes.c_int(param), ctypes.c_int(int(a)), ctypes.c_int(int(w))))


def table_from_func(kind, param, bits) -> np.ndarray:
    n = 1 << bits
    t = np.empty((n, n), dtype=np.int32)
    _check(lib().orc_table_from_func(ctypes.c_int(kind), ctypes.c_int(param), ctypes.c_int(bits), _p(t)), "table_from_func")
    return t


def approx_linear_i16(lut, bits, A, W, threads: int = 1) -> np.ndarray:
    A, W = _i16(A), _i16(W)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    t = np.ascontiguousarray(lut, dtype=np.int32)
    assert t.shape == (1 << bits, 1 << bits)
    acc = np.empty((M, N), dtype=np.int32)
    _check(lib().orc_approx_linear_i16(_p(t), ctypes.c_int(bits), _p(A), _p(W), _p(acc), L(M), L(K), L(N),
                                       ctypes.c_int(threads)), "approx_linear_i16")
    return acc


def approx_linear_func_i16(kind, param, bits, A, W, threads: int = 1) -> np.ndarray:
    A, W = _i16(A), _i16(W)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    _check(lib().orc_approx_linear_func_i16(ctypes.c_int(kind), ctypes.c_int(param), ctypes.c_int(bits), _p(A), _p(W),
                                            _p(acc), L(M), L(K), L(N), ctypes.c_int(threads)), "approx_linear_func_i16")
    return acc


def approx_conv2d_i16(bits, x, w, lut=None, func=None, stride=(1, 1), pad=(0, 0), dil=(1, 1), threads: int = 1) -> np.ndarray:
    """Table form (lut given) or function form (func = (kind, param))."""
    x, w = _i16(x), _i16(w)
    N, Cin, H, W_ = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2 and (lut is None) != (func is None)
    Ho, Wo = conv_out_hw(H, W_, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    acc = np.empty((N, Cout, Ho, Wo), dtype=np.int32)
    t = np.ascontiguousarray(lut, dtype=np.int32) if lut is not None else None
    kind, param = func if func is not None else (0, 0)
    _check(lib().orc_approx_conv2d_i16(_p(t) if t is not None else None, ctypes.c_int(kind), ctypes.c_int(param),
                                       ctypes.c_int(bits), _p(x), _p(w), _p(acc), L(N), L(Cin), L(H), L(W_), L(Cout), L(kh),
                                       L(kw), L(stride[0]), L(stride[1]), L(pad[0]), L(pad[1]), L(dil[0]), L(dil[1]),
                                       ctypes.c_int(threads)), "approx_conv2d_i16")
    return acc


def quantize_i16(x, scale, bits) -> np.ndarray:
    x = _f32(x)
    q = np.empty(x.shape, dtype=np.int16)
    _check(lib().orc_quantize_i16_f32(_p(x), _p(q), ctypes.c_size_t(x.size), ctypes.c_float(float(scale)),
                                      ctypes.c_int(bits)), "quantize_i16")
    return q
