"""GPU parity of grouped convolutions (descriptor field `groups`) against the grouped oracle:
int32 accumulators bit exact, float outputs within 1e-5 relative + 1e-6 absolute."""

import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu

CASES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation, groups
    (1, 1, 1, 2, 1, 1, 2, 1, 0, 1, 2),
    (2, 9, 8, 6, 3, 3, 4, 1, 1, 1, 2),
    (1, 10, 10, 12, 3, 2, 9, 2, 2, 1, 3),
    (2, 14, 14, 64, 3, 3, 64, 1, 1, 1, 32),      # the shape of a 32-group bottleneck
    (2, 16, 16, 32, 3, 3, 48, (2, 1), (1, 2), (1, 2), 4),
    (3, 7, 7, 128, 1, 1, 256, 1, 0, 1, 8),
    (1, 30, 30, 48, 5, 5, 96, 2, 4, 2, 16),      # past the size below which everything is direct anyway
]


def _operands(case, seed, signed):
    N, H, W, Cin, KH, KW, Cout, s, p, d, Gr = case
    rng = np.random.default_rng(seed)
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    x = rng.integers(lo, hi, (N, H, W, Cin)).astype(dt)
    x[rng.random(x.shape) < 0.5] = dt(lo + 5)
    w = rng.integers(lo, hi, (KH, KW, Cin // Gr, Cout)).astype(dt)
    q = I.Quant(0.021, int(rng.integers(lo, hi)), 0.0043, int(rng.integers(lo, hi)),
                None if seed % 2 else int(rng.integers(lo, hi)))
    return x, w, q


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[:7])) + "_g%d" % c[10])
def test_grouped_layers(case, signed):
    s, p, d, Gr = case[7:]
    x, w, q = _operands(case, 50 + case[3] + Gr, signed)
    lut = I.lut_signed_random_error(4) if signed else I.lut_random(6)
    acc, y = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d, groups=Gr)
    torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_grouped(x, w, lut, s, p, q, groups=Gr, dilation=d, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "grouped %r" % (case,))


def test_grouped_layer_through_a_handle_and_from_float():
    case = (2, 14, 14, 32, 3, 3, 64, 1, 1, 1, 4)
    s, p, d, Gr = case[7:]
    x, w, q = _operands(case, 91, False)
    lut = I.lut_random_error(8)
    desc = ax._conv_desc(x.shape, w.shape, s, p, d, False, False, Gr)
    with ax.AxLayer(desc, q) as h:
        assert h.prepared_bytes == 0 and h.workspace_bytes == 0  # direct kernel: nothing prepared
        h.prepare(G.to_dev(w), ax.lut_to_device(lut))
        acc, y = h.run(G.to_dev(x))
        torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_grouped(x, w, lut, s, p, q, groups=Gr, dilation=d)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "handle")
    # float layer: ranges, coefficients and codes as the (separately pinned) quantization oracle
    # gives them, then the grouped oracle on those codes
    rng = np.random.default_rng(92)
    xf = rng.standard_normal(x.shape).astype(np.float32)
    wf = (0.1 * rng.standard_normal(w.shape)).astype(np.float32)
    xr, wr = oracle.range_f32(xf), oracle.range_f32(wf)
    (xa, xb), (wa, wb) = oracle.coeffs(xr), oracle.coeffs(wr)
    xq, wq = oracle.quantize_f32(xf, xa, xb), oracle.quantize_f32(wf, wa, wb)
    qq = I.Quant(xa, xb, wa, wb, None)
    acc_ref, _ = oracle.conv2d_grouped(xq, wq, lut, s, p, qq, groups=Gr, dilation=d)
    acc, y = ax.ax_conv2d_f32_ex(G.to_dev(xf), G.to_dev(wf), ax.lut_to_device(lut), s, p, dilation=d, groups=Gr)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    # y = float(corr) * (alpha1 * alpha2) in float32 on the device; the oracle's y is the double product
    K = 3 * 3 * (32 // Gr)
    Sp_free = oracle.conv2d_grouped(xq, wq, lut, s, p, qq, groups=Gr, dilation=d)[1]
    np.testing.assert_allclose(y.cpu().numpy(), Sp_free, rtol=1e-5, atol=1e-6)


def test_group_errors_are_rejected_on_the_host():
    L = ax.lib()
    D = ax.ax_conv_desc_t
    # Cin not a multiple of the groups; Cout not a multiple; groups together with depthwise; negative
    for d in (D(1, 4, 4, 6, 3, 3, 4, 1, 1, 1, 1, 1, 1, 0, 0, 4), D(1, 4, 4, 6, 3, 3, 4, 1, 1, 1, 1, 1, 1, 0, 0, 3),
              D(1, 4, 4, 4, 3, 3, 4, 1, 1, 1, 1, 1, 1, 1, 0, 2), D(1, 4, 4, 4, 3, 3, 4, 1, 1, 1, 1, 1, 1, 0, 0, -1)):
        assert L.ax_conv2d_ex_workspace_bytes(ctypes.byref(d), None) == 0
    # the backward pass does not take grouped layers
    d = D(1, 4, 4, 4, 3, 3, 4, 1, 1, 1, 1, 1, 1, 0, 0, 2)
    assert L.ax_conv2d_backward_workspace_bytes(ctypes.byref(d)) == 0
    q = ax.ax_quant_t(1.0, 0, 1.0, 0, -1)
    one = ctypes.c_void_p(256)
    assert L.ax_conv2d_backward(ctypes.byref(d), ctypes.byref(q), one, one, one, one, one, one, 1 << 20, None) == -8
