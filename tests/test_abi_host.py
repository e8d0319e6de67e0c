"""Host-side checks that need no GPU: the library builds for gfx950, loads, exports every symbol
the public header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in os.listdir(inc):
        if f.endswith(".h"):
            src = open(os.path.join(inc, f)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(adapt_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    from paper_2203_04071_amd import binding
    return binding.load()


def test_header_declares_the_path():
    names = _declared()
    for must in ("adapt_quantize_f32", "adapt_approx_linear", "adapt_approx_conv2d",
                 "adapt_approx_conv_transpose2d", "adapt_dequant_i32", "adapt_lut_create"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2203_04071_amd import binding
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_bad_arguments_rejected_on_the_host(lib):
    vp = ctypes.c_void_p
    h = vp()
    assert lib.adapt_lut_create(ctypes.byref(h), 9, vp(1)) == -1
    assert b"bits" in lib.adapt_last_error()
    assert lib.adapt_lut_create(ctypes.byref(h), 8, None) == -1
    assert lib.adapt_lut_create(None, 8, vp(1)) == -1
    assert lib.adapt_quantize_f32(vp(16), vp(16), 4, 1.0, 1, None) == -1
    assert lib.adapt_quantize_f32(vp(16), vp(16), 4, 0.0, 8, None) == -1
    assert lib.adapt_quantize_f32(None, vp(16), 4, 1.0, 8, None) == -1
    assert lib.adapt_quantize_f32(None, None, 0, 1.0, 8, None) == 0          # empty is a no-op
    assert lib.adapt_dequant_i32(None, vp(16), 1, 1, 1, 1.0, None, None) == -1
    assert lib.adapt_approx_linear(None, vp(16), vp(16), vp(16), 1, 1, 1, None) == -1
    assert lib.adapt_approx_conv2d(None, vp(16), vp(16), vp(16), 1, 1, 4, 4, 1, 3, 3, 1, 1, 1, 1, 1, 1, 1, None) == -1
    assert lib.adapt_avgpool_hw_f32(vp(16), vp(16), 1, 0, None) == -1
    assert lib.adapt_lstm_cell_f32(None, None, 1.0, 1.0, None, None, None, 2, 2, None) == -1
    assert lib.adapt_lut_destroy(None) == 0


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2203_04071_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "binding" not in text and "libadapt" not in text and "csrc" not in text, f
