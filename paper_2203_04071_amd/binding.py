"""ctypes binding of libadapt_mi355.so: same names as the C ABI (include/adapt_mi355.h),
argument marshalling only.  Tensors are torch CUDA tensors (PyTorch is used for device memory
and streams, nothing else); every step of the path runs in the library's HIP kernels.

There is no CPU fallback: if the library is not built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # imported before the library so that one HIP runtime is shared by both

from . import build as _build

_lib = None

ADAPT_OK = 0
ERRORS = {-1: "INVALID_ARGUMENT", -2: "UNSUPPORTED", -3: "LUT_RANGE", -4: "HIP", -5: "OUT_OF_MEMORY"}

EXPORTS = [
    "adapt_last_error", "adapt_device_cu_count",
    "adapt_lut_create", "adapt_lut_destroy", "adapt_lut_info",
    "adapt_absmax_f32", "adapt_quantize_f32", "adapt_dequant_i32",
    "adapt_absmax_rows_f32", "adapt_quantize_rows_f32", "adapt_dequant_i32_per_channel",
    "adapt_histogram_abs_f32", "adapt_percentile_from_histogram", "adapt_mse_from_histogram", "adapt_entropy_from_histogram",
    "adapt_approx_linear", "adapt_approx_linear_noalloc", "adapt_approx_conv2d", "adapt_approx_conv_transpose2d",
    "adapt_weights_pack_linear", "adapt_weights_pack_conv2d", "adapt_weights_pack_conv_transpose2d",
    "adapt_weights_destroy", "adapt_plan_packed",
    "adapt_approx_linear_packed", "adapt_approx_conv2d_packed", "adapt_approx_conv_transpose2d_packed",
    "adapt_linear_layer_f32", "adapt_conv2d_layer_f32", "adapt_conv_transpose2d_layer_f32",
    "adapt_conv_transpose2d_chain_prepare", "adapt_conv_transpose2d_layer_chain_f32",
    "adapt_conv2d_chain_prepare", "adapt_conv2d_layer_chain_f32", "adapt_conv2d_grouped_layer_f32",
    "adapt_relu_f32", "adapt_add_f32", "adapt_avgpool_hw_f32", "adapt_shortcut_a_f32",
    "adapt_tanh_f32", "adapt_sigmoid_f32", "adapt_lstm_cell_f32", "adapt_lstm_cell_q_f32", "adapt_lstm_step_f32", "adapt_gru_step_f32", "adapt_rnn_step_f32", "adapt_gru_cell_f32", "adapt_rnn_cell_f32",
    "adapt_lut16_create", "adapt_lut16_create_from_func", "adapt_lut16_destroy", "adapt_lut16_bits", "adapt_quantize_i16_f32",
    "adapt_approx_linear_i16", "adapt_approx_conv2d_i16", "adapt_approx_linear_func_i16", "adapt_approx_conv2d_func_i16",
    "adapt_linear_layer_i16_f32", "adapt_conv2d_layer_i16_f32",
    "adapt_ste_linear_backward_f32", "adapt_sgd_step_f32", "adapt_relu_backward_f32", "adapt_ste_conv2d_backward_workspace", "adapt_ste_conv2d_backward_f32",
]


class AdaptError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"adapt_mi355 error {code} ({ERRORS.get(code, '?')}): {text}")
        self.code = code


def lib_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Load the built library (build it first only if nothing is built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    L = ctypes.CDLL(_build.LIB)
    vp, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_float
    L.adapt_last_error.restype = ctypes.c_char_p
    L.adapt_last_error.argtypes = []
    L.adapt_device_cu_count.argtypes = []
    L.adapt_lut_create.argtypes = [ctypes.POINTER(vp), i32, vp]
    L.adapt_lut_destroy.argtypes = [vp]
    L.adapt_lut_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_int32)]
    L.adapt_absmax_f32.argtypes = [vp, sz, vp, vp]
    L.adapt_absmax_rows_f32.argtypes = [vp, sz, sz, vp, vp]
    L.adapt_quantize_rows_f32.argtypes = [vp, vp, sz, sz, vp, i32, vp]
    L.adapt_dequant_i32_per_channel.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp]
    L.adapt_histogram_abs_f32.argtypes = [vp, sz, f32, i32, vp, vp]
    L.adapt_percentile_from_histogram.argtypes = [vp, i32, f32, ctypes.c_uint, ctypes.c_uint, vp, vp]
    L.adapt_mse_from_histogram.argtypes = [vp, i32, f32, i32, vp, vp]
    L.adapt_entropy_from_histogram.argtypes = [vp, i32, f32, i32, vp, vp]
    L.adapt_quantize_f32.argtypes = [vp, vp, sz, f32, i32, vp]
    L.adapt_lut16_create.argtypes = [ctypes.POINTER(vp), i32, vp]
    L.adapt_lut16_create_from_func.argtypes = [ctypes.POINTER(vp), i32, i32, i32]
    L.adapt_lut16_destroy.argtypes = [vp]
    L.adapt_lut16_bits.argtypes = [vp]
    L.adapt_quantize_i16_f32.argtypes = [vp, vp, sz, f32, i32, vp]
    L.adapt_approx_linear_i16.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    L.adapt_approx_conv2d_i16.argtypes = [vp, vp, vp, vp] + [i32] * 13 + [vp]
    L.adapt_approx_linear_func_i16.argtypes = [i32, i32, i32, vp, vp, vp, i32, i32, i32, vp]
    L.adapt_approx_conv2d_func_i16.argtypes = [i32, i32, i32, vp, vp, vp] + [i32] * 13 + [vp]
    L.adapt_linear_layer_i16_f32.argtypes = [vp, i32, i32, i32, vp, vp, vp, i32, i32, i32, f32, f32, vp, vp, i32, vp]
    L.adapt_conv2d_layer_i16_f32.argtypes = [vp, i32, i32, i32, vp, vp, vp] + [i32] * 13 + [f32, f32, vp, vp, i32, vp]
    L.adapt_dequant_i32.argtypes = [vp, vp, sz, sz, sz, f32, vp, vp]
    L.adapt_approx_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    L.adapt_approx_linear_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    L.adapt_approx_conv2d.argtypes = [vp, vp, vp, vp] + [i32] * 14 + [vp]
    L.adapt_approx_conv_transpose2d.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp]
    L.adapt_weights_pack_linear.argtypes = [ctypes.POINTER(vp), vp, vp, i32, i32, vp]
    L.adapt_weights_pack_conv2d.argtypes = [ctypes.POINTER(vp), vp, vp, i32, i32, i32, i32, vp]
    L.adapt_weights_pack_conv_transpose2d.argtypes = [ctypes.POINTER(vp), vp, vp, i32, i32, i32, i32, i32, vp]
    L.adapt_approx_conv_transpose2d_packed.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    L.adapt_weights_destroy.argtypes = [vp]
    L.adapt_plan_packed.argtypes = [i32] * 12 + [ctypes.POINTER(i32)] * 5
    L.adapt_linear_layer_f32.argtypes = [vp, vp, vp, i32, f32, f32, vp, vp, i32, vp]
    L.adapt_conv2d_layer_f32.argtypes = [vp, vp, vp] + [i32] * 9 + [f32, f32, vp, vp, vp, i32, vp]
    L.adapt_conv2d_chain_prepare.argtypes = [vp] + [i32] * 9 + [vp]
    L.adapt_conv2d_grouped_layer_f32.argtypes = [vp, vp, vp, vp] + [i32] * 14 + [f32, f32, vp, vp, i32, vp, f32, vp]
    L.adapt_conv2d_layer_chain_f32.argtypes = [vp, vp, vp] + [i32] * 9 + [f32, f32, vp, vp, vp, i32, vp, f32, vp]
    L.adapt_conv_transpose2d_layer_f32.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, f32, vp, vp, i32, vp]
    L.adapt_conv_transpose2d_chain_prepare.argtypes = [vp, i32, i32, i32, i32, vp]
    L.adapt_conv_transpose2d_layer_chain_f32.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, f32, vp, vp, i32, vp, f32, vp]
    L.adapt_approx_linear_packed.argtypes = [vp, vp, vp, i32, vp]
    L.adapt_approx_conv2d_packed.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
    L.adapt_relu_f32.argtypes = [vp, vp, sz, vp]
    L.adapt_add_f32.argtypes = [vp, vp, vp, sz, i32, vp]
    L.adapt_avgpool_hw_f32.argtypes = [vp, vp, sz, sz, vp]
    L.adapt_shortcut_a_f32.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
    L.adapt_tanh_f32.argtypes = [vp, vp, sz, vp]
    L.adapt_sigmoid_f32.argtypes = [vp, vp, sz, vp]
    L.adapt_lstm_cell_f32.argtypes = [vp, vp, f32, f32, vp, vp, vp, i32, i32, vp]
    L.adapt_lstm_step_f32.argtypes = [vp, vp, vp, f32, f32, f32, vp, vp, vp, vp, i32, i32, vp]
    L.adapt_gru_step_f32.argtypes = [vp, vp, vp, f32, f32, f32, vp, vp, vp, vp, vp, i32, i32, vp]
    L.adapt_rnn_step_f32.argtypes = [vp, vp, vp, f32, f32, f32, vp, i32, vp, vp, i32, i32, vp]
    L.adapt_lstm_cell_q_f32.argtypes = [vp, vp, f32, f32, vp, vp, vp, vp, f32, i32, i32, i32, vp]
    L.adapt_gru_cell_f32.argtypes = [vp, vp, f32, f32, vp, vp, vp, vp, vp, f32, i32, i32, i32, vp]
    L.adapt_rnn_cell_f32.argtypes = [vp, vp, f32, f32, vp, i32, vp, vp, f32, i32, i32, i32, vp]
    L.adapt_sgd_step_f32.argtypes = [vp, vp, sz, f32, vp]
    L.adapt_relu_backward_f32.argtypes = [vp, vp, vp, sz, vp]
    L.adapt_ste_conv2d_backward_workspace.argtypes = [i32] * 15 + [ctypes.POINTER(sz)]
    L.adapt_ste_conv2d_backward_f32.argtypes = [vp, vp, vp] + [i32] * 13 + [f32, f32, i32, vp, vp, vp, vp, sz, vp]
    L.adapt_ste_linear_backward_f32.argtypes = [vp, vp, vp, i32, i32, i32, f32, f32, i32, vp, vp, vp, vp]
    for name in EXPORTS:
        if name != "adapt_last_error":
            getattr(L, name).restype = i32
    _lib = L
    return L


def _chk(rc):
    if rc != ADAPT_OK:
        raise AdaptError(rc, load().adapt_last_error().decode())


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


class Lut:
    """Owner of an adapt_lut handle (multiplier table, Sec. III-C)."""

    def __init__(self, table, bits: int):
        t = np.ascontiguousarray(np.asarray(table, dtype=np.int32))
        if t.size != (1 << bits) ** 2:
            raise ValueError("table must have 2^bits x 2^bits entries")
        self.bits = bits
        self._h = ctypes.c_void_p()
        _chk(load().adapt_lut_create(ctypes.byref(self._h), bits, t.ctypes.data_as(ctypes.c_void_p)))

    @property
    def handle(self):
        return self._h

    def info(self):
        b, s = ctypes.c_int(), ctypes.c_int()
        lo, hi = ctypes.c_int32(), ctypes.c_int32()
        _chk(load().adapt_lut_info(self._h, ctypes.byref(b), ctypes.byref(s), ctypes.byref(lo), ctypes.byref(hi)))
        return dict(bits=b.value, storage=s.value, min=lo.value, max=hi.value)

    def close(self):
        if self._h:
            load().adapt_lut_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def conv_out_hw(H, W, kh, kw, sh, sw, ph, pw, dh=1, dw=1):
    return ((H + 2 * ph - dh * (kh - 1) - 1) // sh + 1, (W + 2 * pw - dw * (kw - 1) - 1) // sw + 1)


class PackedWeights:
    """Owner of an adapt_weights handle (weights of one layer combined with one table)."""

    def __init__(self, lut: Lut, w, kind: str, stream=None, stride: int = 1):
        self._h = ctypes.c_void_p()
        self.kind = kind
        self.shape = tuple(w.shape)
        self.stride = stride
        self._lut = lut         # the library keeps a pointer to the table handle of a transposed-convolution layer
        if kind == "linear":
            N, K = w.shape
            _chk(load().adapt_weights_pack_linear(ctypes.byref(self._h), lut.handle, _ptr(w, torch.int8), K, N,
                                                  _stream(stream)))
        elif kind == "conv2d":
            Cout, Cin, kh, kw = w.shape
            _chk(load().adapt_weights_pack_conv2d(ctypes.byref(self._h), lut.handle, _ptr(w, torch.int8), Cout, Cin,
                                                  kh, kw, _stream(stream)))
        elif kind == "conv_transpose2d":
            Cin, Cout, kh, kw = w.shape
            _chk(load().adapt_weights_pack_conv_transpose2d(ctypes.byref(self._h), lut.handle, _ptr(w, torch.int8), Cin,
                                                            Cout, kh, kw, stride, _stream(stream)))
        else:
            raise ValueError(kind)

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h:
            load().adapt_weights_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def adapt_weights_pack_linear(lut: Lut, w, stream=None) -> PackedWeights:
    return PackedWeights(lut, w, "linear", stream)


def adapt_weights_pack_conv2d(lut: Lut, w, stream=None) -> PackedWeights:
    return PackedWeights(lut, w, "conv2d", stream)


def adapt_weights_pack_conv_transpose2d(lut: Lut, w, stride=1, stream=None) -> PackedWeights:
    return PackedWeights(lut, w, "conv_transpose2d", stream, stride)


def adapt_weights_destroy(pw: PackedWeights):
    pw.close()


def adapt_approx_linear_packed(pw: PackedWeights, a, out=None, stream=None):
    M, K = a.shape
    N, K2 = pw.shape
    assert K == K2 and pw.kind == "linear"
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=a.device)
    _chk(load().adapt_approx_linear_packed(pw.handle, _ptr(a, torch.int8), _ptr(out, torch.int32), M, _stream(stream)))
    return out


def adapt_approx_conv2d_packed(pw: PackedWeights, x, stride=(1, 1), pad=(0, 0), dil=(1, 1), out=None, stream=None):
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = pw.shape
    assert Cin == Cin2 and pw.kind == "conv2d"
    if out is None:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.int32, device=x.device)
    _chk(load().adapt_approx_conv2d_packed(pw.handle, _ptr(x, torch.int8), _ptr(out, torch.int32), N, H, W, stride[0],
                                           stride[1], pad[0], pad[1], dil[0], dil[1], _stream(stream)))
    return out


def adapt_approx_conv_transpose2d_packed(pw: PackedWeights, x, pad=0, out=None, stream=None):
    N, Cin, H, W = x.shape
    Cin2, Cout, kh, kw = pw.shape
    assert Cin == Cin2 and pw.kind == "conv_transpose2d"
    if out is None:
        Ho, Wo = (H - 1) * pw.stride - 2 * pad + kh, (W - 1) * pw.stride - 2 * pad + kw
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.int32, device=x.device)
    _chk(load().adapt_approx_conv_transpose2d_packed(pw.handle, _ptr(x, torch.int8), _ptr(out, torch.int32), N, H, W, pad,
                                                     _stream(stream)))
    return out


def adapt_device_cu_count() -> int:
    n = load().adapt_device_cu_count()
    if n < 0:
        _chk(n)
    return n


def adapt_absmax_f32(x, amax_out=None, stream=None):
    """Returns the 1-element device tensor holding max|x| (no synchronisation)."""
    if amax_out is None:
        amax_out = torch.empty(1, dtype=torch.float32, device=x.device)
    _chk(load().adapt_absmax_f32(_ptr(x, torch.float32), x.numel(), _ptr(amax_out, torch.float32), _stream(stream)))
    return amax_out


def adapt_quantize_f32(x, scale: float, bits: int, out=None, stream=None):
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _chk(load().adapt_quantize_f32(_ptr(x, torch.float32), _ptr(out, torch.int8), x.numel(), float(scale), bits,
                                   _stream(stream)))
    return out


def adapt_dequant_i32(acc, scale: float, outer: int, channels: int, inner: int, bias=None, out=None, stream=None):
    if out is None:
        out = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    assert acc.numel() == outer * channels * inner
    _chk(load().adapt_dequant_i32(_ptr(acc, torch.int32), _ptr(out, torch.float32), outer, channels, inner,
                                  float(scale), _ptr(bias, torch.float32), _stream(stream)))
    return out


def adapt_approx_linear(lut: Lut, a, w, out=None, stream=None):
    M, K = a.shape
    N, K2 = w.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=a.device)
    _chk(load().adapt_approx_linear(lut.handle, _ptr(a, torch.int8), _ptr(w, torch.int8), _ptr(out, torch.int32),
                                    M, K, N, _stream(stream)))
    return out


PLAN_KERNELS = {-1: "lut_rows_kernel", 0: "lut_lines_kernel", 1: "lut_lines_fast_kernel", 2: "lut_lines_fast_kernel (x-major)",
                3: "lut_quad_kernel"}


def adapt_plan_packed(kind, bits, storage, Cout, Cin, kh, kw, stride, rows, Wo, sw, cu=0):
    """(kernel, rows per workgroup, ksplit, steps, workgroups) of a product on a packed handle of this shape."""
    out = [ctypes.c_int() for _ in range(5)]
    _chk(load().adapt_plan_packed(kind, bits, storage, Cout, Cin, kh, kw, stride, rows, Wo, sw, cu, *[ctypes.byref(o) for o in out]))
    return tuple(o.value for o in out)


def adapt_approx_linear_noalloc(lut: Lut, a, w, out, stream=None):
    """The entry point that allocates nothing: `out` ([M][N] int32) is the caller's, as everything else."""
    M, K = a.shape
    N, K2 = w.shape
    assert K == K2 and tuple(out.shape) == (M, N)
    _chk(load().adapt_approx_linear_noalloc(lut.handle, _ptr(a, torch.int8), _ptr(w, torch.int8), _ptr(out, torch.int32),
                                            M, K, N, _stream(stream)))
    return out


def adapt_approx_conv2d(lut: Lut, x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1, out=None, stream=None):
    N, Cin, H, W = x.shape
    Cout, cg, kh, kw = w.shape
    if out is None:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.int32, device=x.device)
    _chk(load().adapt_approx_conv2d(lut.handle, _ptr(x, torch.int8), _ptr(w, torch.int8), _ptr(out, torch.int32),
                                    N, Cin, H, W, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                    groups, _stream(stream)))
    return out


def adapt_approx_conv_transpose2d(lut: Lut, x, w, stride=1, pad=0, out=None, stream=None):
    N, Cin, H, W = x.shape
    Cin2, Cout, kh, kw = w.shape
    assert Cin == Cin2
    if out is None:
        Ho, Wo = (H - 1) * stride - 2 * pad + kh, (W - 1) * stride - 2 * pad + kw
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.int32, device=x.device)
    _chk(load().adapt_approx_conv_transpose2d(lut.handle, _ptr(x, torch.int8), _ptr(w, torch.int8),
                                              _ptr(out, torch.int32), N, Cin, H, W, Cout, kh, kw, stride, pad,
                                              _stream(stream)))
    return out


def adapt_relu_f32(x, out=None, stream=None):
    if out is None:
        out = torch.empty_like(x)
    _chk(load().adapt_relu_f32(_ptr(x, torch.float32), _ptr(out, torch.float32), x.numel(), _stream(stream)))
    return out


def adapt_add_f32(a, b, relu=False, out=None, stream=None):
    assert a.shape == b.shape
    if out is None:
        out = torch.empty_like(a)
    _chk(load().adapt_add_f32(_ptr(a, torch.float32), _ptr(b, torch.float32), _ptr(out, torch.float32), a.numel(),
                              1 if relu else 0, _stream(stream)))
    return out


def adapt_avgpool_hw_f32(x, out=None, stream=None):
    N, C, H, W = x.shape
    if out is None:
        out = torch.empty((N, C), dtype=torch.float32, device=x.device)
    _chk(load().adapt_avgpool_hw_f32(_ptr(x, torch.float32), _ptr(out, torch.float32), N * C, H * W, _stream(stream)))
    return out


def adapt_shortcut_a_f32(x, cout: int, out=None, stream=None):
    N, C, H, W = x.shape
    if out is None:
        out = torch.empty((N, cout, (H + 1) // 2, (W + 1) // 2), dtype=torch.float32, device=x.device)
    _chk(load().adapt_shortcut_a_f32(_ptr(x, torch.float32), _ptr(out, torch.float32), N, C, H, W, cout,
                                     _stream(stream)))
    return out


def adapt_tanh_f32(x, out=None, stream=None):
    if out is None:
        out = torch.empty_like(x)
    _chk(load().adapt_tanh_f32(_ptr(x, torch.float32), _ptr(out, torch.float32), x.numel(), _stream(stream)))
    return out


def adapt_sigmoid_f32(x, out=None, stream=None):
    if out is None:
        out = torch.empty_like(x)
    _chk(load().adapt_sigmoid_f32(_ptr(x, torch.float32), _ptr(out, torch.float32), x.numel(), _stream(stream)))
    return out


def adapt_lstm_cell_f32(acc_ih, acc_hh, s_ih: float, s_hh: float, bias, c, h, stream=None):
    B, H4 = acc_ih.shape
    Hs = H4 // 4
    _chk(load().adapt_lstm_cell_f32(_ptr(acc_ih, torch.int32), _ptr(acc_hh, torch.int32), float(s_ih), float(s_hh),
                                    _ptr(bias, torch.float32), _ptr(c, torch.float32), _ptr(h, torch.float32), B, Hs,
                                    _stream(stream)))
    return h, c


def adapt_lstm_cell_q_f32(acc_ih, acc_hh, s_ih: float, s_hh: float, bias, c, h, qh, s_h: float, bits: int, stream=None):
    B, H4 = acc_ih.shape
    Hs = H4 // 4
    _chk(load().adapt_lstm_cell_q_f32(_ptr(acc_ih, torch.int32), _ptr(acc_hh, torch.int32), float(s_ih), float(s_hh),
                                      _ptr(bias, torch.float32), _ptr(c, torch.float32), _ptr(h, torch.float32),
                                      _ptr(qh, torch.int8), float(s_h), bits, B, Hs, _stream(stream)))
    return h, c, qh


def adapt_gru_cell_f32(acc_ih, acc_hh, s_ih: float, s_hh: float, b_ih, b_hh, h_prev, h, qh=None, s_h: float = 1.0, bits: int = 8,
                       stream=None):
    B, H3 = acc_ih.shape
    Hs = H3 // 3
    _chk(load().adapt_gru_cell_f32(_ptr(acc_ih, torch.int32), _ptr(acc_hh, torch.int32), float(s_ih), float(s_hh),
                                   _ptr(b_ih, torch.float32), _ptr(b_hh, torch.float32), _ptr(h_prev, torch.float32),
                                   _ptr(h, torch.float32), _ptr(qh, torch.int8), float(s_h), bits, B, Hs, _stream(stream)))
    return h, qh


def adapt_rnn_cell_f32(acc_ih, acc_hh, s_ih: float, s_hh: float, bias, h, relu: bool = False, qh=None, s_h: float = 1.0,
                       bits: int = 8, stream=None):
    B, Hs = acc_ih.shape
    _chk(load().adapt_rnn_cell_f32(_ptr(acc_ih, torch.int32), _ptr(acc_hh, torch.int32), float(s_ih), float(s_hh),
                                   _ptr(bias, torch.float32), 1 if relu else 0, _ptr(h, torch.float32), _ptr(qh, torch.int8),
                                   float(s_h), bits, B, Hs, _stream(stream)))
    return h, qh


# ---- operands wider than 8 bits, multipliers as functions (Sec. III-C)

FUNC_EXACT, FUNC_TRUNC, FUNC_MITCHELL = 0, 1, 2


class Lut16:
    """Owner of an adapt_lut16 handle: a 2^bits x 2^bits int32 table in device memory (bits <= 12), from a host table or
    generated on the device from a function-described multiplier (func = (kind, param))."""

    def __init__(self, bits: int, table=None, func=None):
        assert (table is None) != (func is None)
        self.bits = bits
        self._h = ctypes.c_void_p()
        if table is not None:
            t = np.ascontiguousarray(np.asarray(table, dtype=np.int32))
            if t.size != (1 << bits) ** 2:
                raise ValueError("table must have 2^bits x 2^bits entries")
            _chk(load().adapt_lut16_create(ctypes.byref(self._h), bits, t.ctypes.data_as(ctypes.c_void_p)))
        else:
            _chk(load().adapt_lut16_create_from_func(ctypes.byref(self._h), func[0], func[1], bits))

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h:
            load().adapt_lut16_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def adapt_quantize_i16_f32(x, scale: float, bits: int, out=None, stream=None):
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int16, device=x.device)
    _chk(load().adapt_quantize_i16_f32(_ptr(x, torch.float32), _ptr(out, torch.int16), x.numel(), float(scale), bits,
                                       _stream(stream)))
    return out


def adapt_approx_linear_i16(lut: Lut16, a, w, out=None, stream=None):
    M, K = a.shape
    N, K2 = w.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=a.device)
    _chk(load().adapt_approx_linear_i16(lut.handle, _ptr(a, torch.int16), _ptr(w, torch.int16), _ptr(out, torch.int32), M, K, N,
                                        _stream(stream)))
    return out


def adapt_approx_linear_func_i16(kind: int, param: int, bits: int, a, w, out=None, stream=None):
    M, K = a.shape
    N, K2 = w.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=a.device)
    _chk(load().adapt_approx_linear_func_i16(kind, param, bits, _ptr(a, torch.int16), _ptr(w, torch.int16),
                                             _ptr(out, torch.int32), M, K, N, _stream(stream)))
    return out


def _conv_i16_out(x, w, stride, pad, dil, out):
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2
    if out is None:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.int32, device=x.device)
    return out, (N, Cin, H, W, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])


def adapt_approx_conv2d_i16(lut: Lut16, x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), out=None, stream=None):
    out, dims = _conv_i16_out(x, w, stride, pad, dil, out)
    _chk(load().adapt_approx_conv2d_i16(lut.handle, _ptr(x, torch.int16), _ptr(w, torch.int16), _ptr(out, torch.int32), *dims,
                                        _stream(stream)))
    return out


def adapt_approx_conv2d_func_i16(kind: int, param: int, bits: int, x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), out=None,
                                 stream=None):
    out, dims = _conv_i16_out(x, w, stride, pad, dil, out)
    _chk(load().adapt_approx_conv2d_func_i16(kind, param, bits, _ptr(x, torch.int16), _ptr(w, torch.int16),
                                             _ptr(out, torch.int32), *dims, _stream(stream)))
    return out


ACT_NONE, ACT_RELU, ACT_TANH = 0, 1, 2


def _scales(s_out):
    """(scalar, vector) forms of an output scale: a tensor means one scale per channel."""
    if isinstance(s_out, torch.Tensor):
        return 1.0, _ptr(s_out, torch.float32)
    return float(s_out), None


def adapt_linear_layer_i16_f32(mul, x, w, s_x, s_out, bias=None, act=ACT_NONE, out=None, stream=None):
    """mul: a Lut16 (table form) or a tuple (kind, param, bits) (function form)."""
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=x.device)
    lut, (kind, param, bits) = (mul.handle, (0, 0, 0)) if isinstance(mul, Lut16) else (None, mul)
    sc, sv = _scales(s_out)
    _chk(load().adapt_linear_layer_i16_f32(lut, kind, param, bits, _ptr(x, torch.float32), _ptr(w, torch.int16), _ptr(out, torch.float32),
                                           M, K, N, float(s_x), sc, sv, _ptr(bias, torch.float32), act, _stream(stream)))
    return out


def adapt_conv2d_layer_i16_f32(mul, x, w, s_x, s_out, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None, act=ACT_NONE, out=None, stream=None):
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2
    if out is None:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.float32, device=x.device)
    lut, (kind, param, bits) = (mul.handle, (0, 0, 0)) if isinstance(mul, Lut16) else (None, mul)
    sc, sv = _scales(s_out)
    _chk(load().adapt_conv2d_layer_i16_f32(lut, kind, param, bits, _ptr(x, torch.float32), _ptr(w, torch.int16), _ptr(out, torch.float32),
                                           N, Cin, H, W, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                           float(s_x), sc, sv, _ptr(bias, torch.float32), act, _stream(stream)))
    return out


def adapt_linear_layer_f32(pw: PackedWeights, x, s_x, s_out, bias=None, act=ACT_NONE, out=None, stream=None):
    M, K = x.shape
    N, K2 = pw.shape
    assert K == K2 and pw.kind == "linear"
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=x.device)
    sc, sv = _scales(s_out)
    _chk(load().adapt_linear_layer_f32(pw.handle, _ptr(x, torch.float32), _ptr(out, torch.float32), M, float(s_x), sc, sv,
                                       _ptr(bias, torch.float32), act, _stream(stream)))
    return out


def adapt_conv2d_layer_f32(pw: PackedWeights, x, s_x, s_out, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None, act=ACT_NONE,
                           out=None, stream=None, residual=None):
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = pw.shape
    assert Cin == Cin2 and pw.kind == "conv2d"
    if out is None:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.float32, device=x.device)
    sc, sv = _scales(s_out)
    _chk(load().adapt_conv2d_layer_f32(pw.handle, _ptr(x, torch.float32), _ptr(out, torch.float32), N, H, W, stride[0], stride[1],
                                       pad[0], pad[1], dil[0], dil[1], float(s_x), sc, sv, _ptr(bias, torch.float32),
                                       _ptr(residual, torch.float32), act, _stream(stream)))
    return out


def adapt_conv2d_chain_prepare(pw: PackedWeights, N, H, W, stride=(1, 1), pad=(0, 0), dil=(1, 1), stream=None):
    assert pw.kind == "conv2d"
    _chk(load().adapt_conv2d_chain_prepare(pw.handle, N, H, W, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], _stream(stream)))


def adapt_conv2d_layer_chain_f32(pw: PackedWeights, x, s_x, s_out, out, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None,
                                 act=ACT_NONE, residual=None, next_pw: PackedWeights = None, s_next: float = 1.0, in_shape=None,
                                 stream=None):
    """x None: the input copy is already in pw's prepared workspace (in_shape = (N, H, W) then); next_pw: also write the
    output as next_pw's input copy, quantised with s_next.  `out` (fp32 [N][Cout][Ho][Wo]) may be None when next_pw is given and
    only that copy is wanted; shapes that finish their sums in a separate pass then raise AdaptError with code -2."""
    if x is not None:
        N, Cin, H, W = x.shape
    else:
        N, H, W = in_shape
    s_scalar, s_vec = _scales(s_out)
    _chk(load().adapt_conv2d_layer_chain_f32(pw.handle, _ptr(x, torch.float32), _ptr(out, torch.float32), N, H, W, stride[0], stride[1],
                                             pad[0], pad[1], dil[0], dil[1], float(s_x), s_scalar, s_vec, _ptr(bias, torch.float32),
                                             _ptr(residual, torch.float32), act, next_pw.handle if next_pw is not None else None,
                                             float(s_next), _stream(stream)))
    return out


def adapt_conv2d_grouped_layer_f32(lut: Lut, x, w, s_x, s_out, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1, bias=None, act=ACT_NONE,
                                   out=None, want_out=True, next_pw: PackedWeights = None, s_next: float = 1.0, stream=None):
    """Grouped convolution as one call (fp32 in; fp32 out and / or the next layer's input copy): one kernel for groups of fewer than
    8 output channels, quantiser + whole-table kernel for larger groups (these need the fp32 output)."""
    N, Cin, H, W = x.shape
    Cout, cg, kh, kw = w.shape
    if out is None and want_out:
        Ho, Wo = conv_out_hw(H, W, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.float32, device=x.device)
    s_scalar, s_vec = _scales(s_out)
    _chk(load().adapt_conv2d_grouped_layer_f32(lut.handle, _ptr(x, torch.float32), _ptr(w, torch.int8), _ptr(out, torch.float32), N, Cin,
                                               H, W, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], groups,
                                               float(s_x), s_scalar, s_vec, _ptr(bias, torch.float32), act,
                                               next_pw.handle if next_pw is not None else None, float(s_next), _stream(stream)))
    return out


def adapt_conv_transpose2d_layer_f32(pw: PackedWeights, x, s_x, s_out, pad=0, bias=None, act=ACT_NONE, out=None, stream=None):
    N, Cin, H, W = x.shape
    Cin2, Cout, kh, kw = pw.shape
    assert Cin == Cin2 and pw.kind == "conv_transpose2d"
    if out is None:
        Ho, Wo = (H - 1) * pw.stride - 2 * pad + kh, (W - 1) * pw.stride - 2 * pad + kw
        out = torch.empty((N, Cout, Ho, Wo), dtype=torch.float32, device=x.device)
    sc, sv = _scales(s_out)
    _chk(load().adapt_conv_transpose2d_layer_f32(pw.handle, _ptr(x, torch.float32), _ptr(out, torch.float32), N, H, W, pad,
                                                 float(s_x), sc, sv, _ptr(bias, torch.float32), act, _stream(stream)))
    return out


def adapt_conv_transpose2d_chain_prepare(pw: PackedWeights, N, H, W, pad=0, stream=None):
    """Raises AdaptError with code -2 (UNSUPPORTED) for geometries outside the phase form."""
    assert pw.kind == "conv_transpose2d"
    _chk(load().adapt_conv_transpose2d_chain_prepare(pw.handle, N, H, W, pad, _stream(stream)))


def adapt_conv_transpose2d_layer_chain_f32(pw: PackedWeights, x, s_x, s_out, out, pad=0, bias=None, act=ACT_NONE,
                                           next_pw: PackedWeights = None, s_next: float = 1.0, in_shape=None, stream=None):
    """x None: the input copy is already in pw's prepared workspace (in_shape = (N, H, W) then); next_pw: also write the
    output as next_pw's input copy, quantised with s_next.  `out` (fp32 [N][Cout][Ho][Wo]) may be None when next_pw is given and
    only that copy is wanted; shapes that finish their sums in a separate pass then raise AdaptError with code -2."""
    if x is not None:
        N, Cin, H, W = x.shape
    else:
        N, H, W = in_shape
    sc, sv = _scales(s_out)
    _chk(load().adapt_conv_transpose2d_layer_chain_f32(pw.handle, _ptr(x, torch.float32), _ptr(out, torch.float32), N, H, W, pad,
                                                       float(s_x), sc, sv, _ptr(bias, torch.float32), act,
                                                       next_pw.handle if next_pw is not None else None, float(s_next), _stream(stream)))
    return out


def adapt_lstm_step_f32(pw_hh: PackedWeights, qh, acc_ih, s_ih, s_hh, s_h, bias, c, h, qh_next, stream=None):
    """Raises AdaptError with code -2 (UNSUPPORTED) when the shape does not fit the fused kernel."""
    B, H4 = acc_ih.shape
    Hs = H4 // 4
    _chk(load().adapt_lstm_step_f32(pw_hh.handle, _ptr(qh, torch.int8), _ptr(acc_ih, torch.int32), float(s_ih), float(s_hh),
                                    float(s_h), _ptr(bias, torch.float32), _ptr(c, torch.float32), _ptr(h, torch.float32),
                                    _ptr(qh_next, torch.int8), B, Hs, _stream(stream)))
    return h, c, qh_next


def adapt_gru_step_f32(pw_hh: PackedWeights, qh, acc_ih, s_ih, s_hh, s_h, b_ih, b_hh, h_prev, h, qh_next, stream=None):
    """Raises AdaptError with code -2 (UNSUPPORTED) when the shape does not fit the fused kernel."""
    B, H3 = acc_ih.shape
    Hs = H3 // 3
    _chk(load().adapt_gru_step_f32(pw_hh.handle, _ptr(qh, torch.int8), _ptr(acc_ih, torch.int32), float(s_ih), float(s_hh),
                                   float(s_h), _ptr(b_ih, torch.float32), _ptr(b_hh, torch.float32), _ptr(h_prev, torch.float32),
                                   _ptr(h, torch.float32), _ptr(qh_next, torch.int8), B, Hs, _stream(stream)))
    return h, qh_next


def adapt_rnn_step_f32(pw_hh: PackedWeights, qh, acc_ih, s_ih, s_hh, s_h, bias, h, qh_next, relu=False, stream=None):
    """Raises AdaptError with code -2 (UNSUPPORTED) when the shape does not fit the fused kernel."""
    B, Hs = acc_ih.shape
    _chk(load().adapt_rnn_step_f32(pw_hh.handle, _ptr(qh, torch.int8), _ptr(acc_ih, torch.int32), float(s_ih), float(s_hh),
                                   float(s_h), _ptr(bias, torch.float32), 1 if relu else 0, _ptr(h, torch.float32),
                                   _ptr(qh_next, torch.int8), B, Hs, _stream(stream)))
    return h, qh_next


def adapt_absmax_rows_f32(x, out=None, stream=None):
    rows = x.shape[0]
    cols = x.numel() // rows if rows else 0
    if out is None:
        out = torch.empty((rows,), dtype=torch.float32, device=x.device)
    _chk(load().adapt_absmax_rows_f32(_ptr(x, torch.float32), rows, cols, _ptr(out, torch.float32), _stream(stream)))
    return out


def adapt_quantize_rows_f32(x, scales, bits, out=None, stream=None):
    rows = x.shape[0]
    cols = x.numel() // rows
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _chk(load().adapt_quantize_rows_f32(_ptr(x, torch.float32), _ptr(out, torch.int8), rows, cols, _ptr(scales, torch.float32),
                                        bits, _stream(stream)))
    return out


def adapt_dequant_i32_per_channel(acc, scales, outer, channels, inner, bias=None, out=None, stream=None):
    if out is None:
        out = torch.empty(acc.shape, dtype=torch.float32, device=acc.device)
    _chk(load().adapt_dequant_i32_per_channel(_ptr(acc, torch.int32), _ptr(out, torch.float32), outer, channels, inner,
                                              _ptr(scales, torch.float32), _ptr(bias, torch.float32), _stream(stream)))
    return out


def adapt_histogram_abs_f32(x, amax, bins, counts=None, stream=None):
    """counts (int32 tensor holding uint32 counters) is accumulated into; a new one starts at zero."""
    if counts is None:
        counts = torch.zeros((bins,), dtype=torch.int32, device=x.device)
    _chk(load().adapt_histogram_abs_f32(_ptr(x, torch.float32), x.numel(), float(amax), bins, _ptr(counts, torch.int32),
                                        _stream(stream)))
    return counts


def adapt_percentile_from_histogram(counts, amax, num=999, den=1000, out=None, stream=None):
    if out is None:
        out = torch.empty((1,), dtype=torch.float32, device=counts.device)
    _chk(load().adapt_percentile_from_histogram(_ptr(counts, torch.int32), counts.numel(), float(amax), num, den,
                                                _ptr(out, torch.float32), _stream(stream)))
    return out


def adapt_mse_from_histogram(counts, amax, bits, out=None, stream=None):
    if out is None:
        out = torch.empty((1,), dtype=torch.float32, device=counts.device)
    _chk(load().adapt_mse_from_histogram(_ptr(counts, torch.int32), counts.numel(), float(amax), bits, _ptr(out, torch.float32),
                                         _stream(stream)))
    return out



def adapt_entropy_from_histogram(counts, amax, bits, out=None, stream=None):
    if out is None:
        out = torch.empty((1,), dtype=torch.float32, device=counts.device)
    _chk(load().adapt_entropy_from_histogram(_ptr(counts, torch.int32), counts.numel(), float(amax), bits, _ptr(out, torch.float32),
                                             _stream(stream)))
    return out


def adapt_ste_linear_backward_f32(dy, x, w, s_x, s_w, bits, want=("dx", "dw", "db"), out=None, stream=None):
    """dy [M][N], x [M][K], w [N][K] fp32 -> (dx, dw, db); entries not named in `want` are None.
    out: (dx, dw, db) tensors to write into (None entries are not computed) instead of new ones."""
    M, N = dy.shape
    K = x.shape[1]
    assert x.shape == (M, K) and w.shape == (N, K)
    if out is not None:
        dx, dw, db = out
        assert (dx is None or dx.shape == (M, K)) and (dw is None or dw.shape == (N, K)) and (db is None or db.shape == (N,))
    else:
        dx = torch.empty((M, K), dtype=torch.float32, device=dy.device) if "dx" in want else None
        dw = torch.empty((N, K), dtype=torch.float32, device=dy.device) if "dw" in want else None
        db = torch.empty((N,), dtype=torch.float32, device=dy.device) if "db" in want else None
    _chk(load().adapt_ste_linear_backward_f32(_ptr(dy, torch.float32), _ptr(x, torch.float32), _ptr(w, torch.float32), M, K, N,
                                              float(s_x), float(s_w), int(bits), _ptr(dx, torch.float32), _ptr(dw, torch.float32),
                                              _ptr(db, torch.float32), _stream(stream)))
    return dx, dw, db


def adapt_sgd_step_f32(w, g, lr, stream=None):
    """w <- w - lr * g in place."""
    assert w.shape == g.shape
    _chk(load().adapt_sgd_step_f32(_ptr(w, torch.float32), _ptr(g, torch.float32), w.numel(), float(lr), _stream(stream)))
    return w


def adapt_ste_conv2d_backward_f32(dy, x, w, stride, pad, dil, s_x, s_w, bits, want=("dx", "dw", "db"), workspace=None, stream=None):
    """dy [N][Cout][Ho][Wo], x [N][Cin][H][W], w [Cout][Cin][kh][kw] fp32 -> (dx, dw, db); entries not in `want` are None.
    workspace: a uint8 device tensor to reuse (allocated here when None or too small)."""
    N, Cin, H, W = x.shape
    Cout, Cin2, kh, kw = w.shape
    assert Cin == Cin2 and dy.shape[:2] == (N, Cout)
    geo = (N, Cin, H, W, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])
    need = ctypes.c_size_t(0)
    _chk(load().adapt_ste_conv2d_backward_workspace(*geo, 1 if "dx" in want else 0, 1 if "dw" in want else 0, ctypes.byref(need)))
    if workspace is None or workspace.numel() < need.value:
        workspace = torch.empty(max(need.value, 256), dtype=torch.uint8, device=x.device)
    dx = torch.empty_like(x) if "dx" in want else None
    dw = torch.empty_like(w) if "dw" in want else None
    db = torch.empty((Cout,), dtype=torch.float32, device=x.device) if "db" in want else None
    _chk(load().adapt_ste_conv2d_backward_f32(_ptr(dy, torch.float32), _ptr(x, torch.float32), _ptr(w, torch.float32), *geo, float(s_x),
                                              float(s_w), int(bits), _ptr(dx, torch.float32), _ptr(dw, torch.float32),
                                              _ptr(db, torch.float32), ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                              _stream(stream)))
    return dx, dw, db


def adapt_relu_backward_f32(dy, y, out=None, stream=None):
    """dy where y > 0, else 0 (out may be dy)."""
    assert dy.shape == y.shape
    if out is None:
        out = torch.empty_like(dy)
    _chk(load().adapt_relu_backward_f32(_ptr(dy, torch.float32), _ptr(y, torch.float32), _ptr(out, torch.float32), dy.numel(), _stream(stream)))
    return out
