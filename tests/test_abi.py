"""The C-ABI library loads and exports every function include/axconv.h declares (CPU only:
no compute call is made)."""

import ctypes
import os
import re

import pytest

from paper_2002_09481_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "axconv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ax_[a-z0-9_]+)\s*\(", src)))


def test_header_functions_are_exported():
    names = _declared()
    assert "ax_conv2d" in names and "ax_dense" in names and len(names) >= 8
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libaxconv.so not built")
    L = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_host_side_calls_without_gpu():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libaxconv.so not built")
    assert binding.ax_version() >= 100
    assert binding.ax_strerror(0) == "ok" and "NULL" in binding.ax_strerror(-1)
    binding.ax_set_option("variant", 1)
    assert binding.ax_get_option("variant") == 1
    binding.ax_set_option("variant", 0)
    with pytest.raises(binding.AxError):
        binding.ax_set_option("variant", 99)
    with pytest.raises(binding.AxError):
        binding.ax_set_option("no_such_option", 1)
    for name, top in (("share_order", 2), ("timing", 16), ("row_tiles", 1 << 20)):
        binding.ax_set_option(name, top)
        assert binding.ax_get_option(name) == top
        with pytest.raises(binding.AxError):
            binding.ax_set_option(name, top + 1)
        binding.ax_set_option(name, 0)
    # workspace queries are pure host arithmetic
    assert binding.ax_conv2d_workspace_bytes((1, 16, 16, 8), (3, 3, 8, 8), 1, 1) >= 256
    assert binding.ax_dense_workspace_bytes(32, 2048, 1000) >= 256
    assert binding.ax_conv2d_workspace_bytes((1, 2, 2, 8), (3, 3, 8, 8), 1, 0) == 0  # empty output
    # argument validation happens before anything touches a device
    L = binding.lib()
    q = binding.ax_quant_t(1.0, 0, 1.0, 0, -1)
    one = ctypes.c_void_p(256)
    assert L.ax_dense(None, 1, 1, one, 1, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -1
    assert L.ax_dense(one, 0, 1, one, 1, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -2
    assert L.ax_dense(one, 1, 40000, one, 1, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -4
    bad = binding.ax_quant_t(1.0, 300, 1.0, 0, -1)
    assert L.ax_dense(one, 1, 1, one, 1, one, ctypes.byref(bad), one, one, one, 1 << 20, None) == -3
    bad = binding.ax_quant_t(float("nan"), 0, 1.0, 0, -1)
    assert L.ax_dense(one, 1, 1, one, 1, one, ctypes.byref(bad), one, one, one, 1 << 20, None) == -3
    assert L.ax_dense(one, 1, 1, one, 1, ctypes.c_void_p(257), ctypes.byref(q), one, one, one, 1 << 20, None) == -7


def test_host_side_validation_of_the_later_entry_points():
    """Descriptor, table-count, range and float-layer entry points reject bad arguments on the
    host, before any device work."""
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libaxconv.so not built")
    L = binding.lib()
    one = ctypes.c_void_p(256)
    q = binding.ax_quant_t(1.0, 0, 1.0, 0, -1)
    D = binding.ax_conv_desc_t
    ok = D(1, 8, 8, 16, 3, 3, 16, 1, 1, 1, 1, 1, 1, 0, 0)
    assert L.ax_conv2d_ex_workspace_bytes(ctypes.byref(ok)) >= 256
    assert L.ax_conv2d_ex(None, one, one, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -1
    bad_dil = D(1, 8, 8, 16, 3, 3, 16, 1, 1, 1, 1, 0, 1, 0, 0)
    assert L.ax_conv2d_ex(ctypes.byref(bad_dil), one, one, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -2
    too_wide = D(1, 8, 8, 16, 3, 3, 16, 1, 1, 1, 1, 5, 5, 0, 0)  # dilated kernel larger than the padded image
    assert L.ax_conv2d_ex_workspace_bytes(ctypes.byref(too_wide)) == 0
    bad_flag = D(1, 8, 8, 16, 3, 3, 16, 1, 1, 1, 1, 1, 1, 0, 3)
    assert L.ax_conv2d_ex(ctypes.byref(bad_flag), one, one, one, ctypes.byref(q), one, one, one, 1 << 20, None) == -8
    bad_dw = D(1, 8, 8, 16, 3, 3, 24, 1, 1, 1, 1, 1, 1, 1, 0)  # Cout not a multiple of Cin
    assert L.ax_conv2d_ex_workspace_bytes(ctypes.byref(bad_dw)) == 0
    signed = D(1, 8, 8, 16, 3, 3, 16, 1, 1, 1, 1, 1, 1, 0, 1)
    qs = binding.ax_quant_t(1.0, -128, 1.0, 127, binding.AX_PAD_DEFAULT)
    assert L.ax_conv2d_ex(ctypes.byref(signed), None, one, one, ctypes.byref(qs), one, one, one, 1 << 20, None) == -1
    qbad = binding.ax_quant_t(1.0, 128, 1.0, 0, binding.AX_PAD_DEFAULT)  # 128 is no signed code
    assert L.ax_conv2d_ex(ctypes.byref(signed), one, one, one, ctypes.byref(qbad), one, one, one, 1 << 20, None) == -3
    # table counts
    assert binding.ax_conv2d_multi_lut_workspace_bytes((1, 8, 8, 16), (3, 3, 16, 16), 4, 1, 1) >= 4 * 131072
    assert L.ax_conv2d_multi_lut_workspace_bytes(1, 8, 8, 16, 3, 3, 16, 0, 1, 1, 1, 1) == 0
    assert L.ax_conv2d_multi_lut(one, 1, 8, 8, 16, one, 3, 3, 16, one, 0, 1, 1, 1, 1, ctypes.byref(q), one, one, one,
                                 1 << 30, None) == -2
    # float side
    assert binding.ax_range_workspace_bytes(1000) >= 256
    assert L.ax_range_f32(one, 0, 0, one, one, 1 << 20, None) == -2
    assert L.ax_range_f32(one, 8, 0, one, one, 16, None) == -5
    assert L.ax_quantize_f32(one, 8, one, 0, 7, one, None, None) == -8
    assert L.ax_quantize_f32(ctypes.c_void_p(258), 8, one, 0, 0, one, None, None) == -7
    assert binding.ax_conv2d_f32_workspace_bytes((1, 8, 8, 16), (3, 3, 16, 16), 1, 1) > \
        binding.ax_conv2d_workspace_bytes((1, 8, 8, 16), (3, 3, 16, 16), 1, 1)
    assert L.ax_conv2d_f32(one, 1, 8, 8, 16, one, 3, 3, 16, one, 1, 1, 1, 1, None, None, 0, 2, one, one, one, 1 << 30,
                           None) == -8
    assert L.ax_conv2d_f32(one, 1, 8, 8, 16, one, 3, 3, 16, one, 1, 1, 1, 1, None, None, 0, 0, one, one, one, 16,
                           None) == -5
    assert L.ax_conv2d_f32_ex(None, one, one, one, None, None, 0, 0, one, one, one, 1 << 30, None) == -1
    assert L.ax_conv2d_f32_ex_workspace_bytes(ctypes.byref(signed)) > 0
    assert binding.ax_version() >= 200
