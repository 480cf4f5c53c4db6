"""GPU parity of transposed convolutions (ax_conv2d_transpose) against the transposed oracle:
int32 accumulators bit exact, float outputs within 1e-5 relative + 1e-6 absolute, through every
kernel family the inner stride-1 layer can take."""

import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    ax.ax_set_option("variant", 0)


CASES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation
    (1, 1, 1, 1, 1, 1, 1, 1, 0, 1),
    (2, 5, 4, 3, 3, 3, 4, 2, 1, 1),
    (1, 6, 6, 2, 2, 2, 3, 2, 0, 1),
    (2, 4, 5, 4, 3, 2, 2, (3, 2), (1, 0), 1),
    (1, 4, 4, 2, 3, 3, 3, 2, 2, 2),
    (2, 14, 14, 32, 3, 3, 48, 2, 1, 1),     # table-tile kernels, implicit patch view
    (1, 20, 20, 20, 4, 4, 24, 2, 1, 1),     # the usual 4 x 4 stride-2 upsampling layer, materialized patches
    (2, 7, 7, 256, 2, 2, 128, 2, 0, 1),     # many channels
]


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "x".join(map(str, c[:7])) + "_s%s" % (c[7],))
def test_transposed_layers(case, signed, variant):
    N, H, W, Cin, KH, KW, Cout, s, p, d = case
    rng = np.random.default_rng(600 + H + Cin)
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    x = rng.integers(lo, hi, (N, H, W, Cin)).astype(dt)
    w = rng.integers(lo, hi, (KH, KW, Cin, Cout)).astype(dt)
    q = I.Quant(0.021, int(rng.integers(lo, hi)), 0.0043, int(rng.integers(lo, hi)),
                None if (H + Cin) % 2 else int(rng.integers(lo, hi)))
    lut = I.lut_signed_random_error(4) if signed else I.lut_random(6)
    ax.ax_set_option("variant", variant)
    acc, y = ax.ax_conv2d_transpose(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d)
    torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_transpose(x, w, lut, s, p, q, dilation=d, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "transposed %r variant %d" % (case, variant))


def test_transposed_descriptor_errors_are_rejected_on_the_host():
    L = ax.lib()
    D = ax.ax_conv_desc_t
    one = ctypes.c_void_p(256)
    q = ax.ax_quant_t(1.0, 0, 1.0, 0, -1)
    # padding beyond what the filter reaches; depthwise; groups
    for d in (D(1, 4, 4, 2, 3, 3, 2, 2, 2, 3, 3, 1, 1, 0, 0, 0), D(1, 4, 4, 2, 3, 3, 2, 2, 2, 1, 1, 1, 1, 1, 0, 0),
              D(1, 4, 4, 2, 3, 3, 2, 2, 2, 1, 1, 1, 1, 0, 0, 2)):
        assert L.ax_conv2d_transpose_workspace_bytes(ctypes.byref(d), None) == 0
        assert L.ax_conv2d_transpose(ctypes.byref(d), None, one, one, one, ctypes.byref(q), one, one, one, 1 << 30, None) < 0
    d = D(1, 4, 4, 2, 3, 3, 2, 2, 2, 1, 1, 1, 1, 0, 0, 0)
    n = L.ax_conv2d_transpose_workspace_bytes(ctypes.byref(d), None)
    assert n > 0
    # workspace too small or missing: rejected before anything is launched
    assert L.ax_conv2d_transpose(ctypes.byref(d), None, one, one, one, ctypes.byref(q), one, one, one, n - 1, None) == -5
    assert L.ax_conv2d_transpose(ctypes.byref(d), None, one, one, one, ctypes.byref(q), one, one, None, 0, None) == -5
