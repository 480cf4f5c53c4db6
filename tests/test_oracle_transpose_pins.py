"""Pins of the transposed-convolution oracle against things other than itself (CPU only): a hand
case, the float64 transposed convolution of the library on the dequantized tensors (exact table),
and the already pinned ordinary oracle on an input that is spread out explicitly, with the filters
flipped (arbitrary tables, inserted positions and pad codes included)."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I


def test_hand_case():
    """One channel, x = [1, 2] (1 x 2 image), filter [3, 4] (1 x 2), stride 2, no padding, exact
    table, zero points 0: output = [1*3, 1*4, 2*3, 2*4] ... with the stride-2 placement
    oy = 0; ox = ix*2 + kx: [3, 4, 6, 8]."""
    x = np.array([1, 2], np.uint8).reshape(1, 1, 2, 1)
    w = np.array([3, 4], np.uint8).reshape(1, 2, 1, 1)
    acc, y = oracle.conv2d_transpose(x, w, I.lut_exact(), (1, 2), 0, I.Quant(1.0, 0, 1.0, 0, -1))
    assert acc.shape == (1, 1, 4, 1)
    assert acc.reshape(-1).tolist() == [3, 4, 6, 8] and y.reshape(-1).tolist() == [3.0, 4.0, 6.0, 8.0]
    # a table that returns 1 for every pair counts the taps: every output has KH*KW*Cin = 2 of them,
    # on pixels, on inserted positions or outside
    ones = np.ones(65536, np.uint16)
    acc, _ = oracle.conv2d_transpose(x, w, ones, (1, 2), 0, I.Quant(1.0, 0, 1.0, 0, -1))
    assert acc.reshape(-1).tolist() == [2, 2, 2, 2]
    # a table that returns the activation code shows which code each tap fed: zero point 7 on the
    # inserted position (between the two pixels), pad code 9 outside
    first = np.repeat(np.arange(256, dtype=np.uint16), 256)
    acc, _ = oracle.conv2d_transpose(x, w, first, (1, 2), 0, I.Quant(1.0, 7, 1.0, 0, 9))
    # ox=0: taps at positions 0 (pixel 1) and -1 (outside: 9); ox=1: 1 (inserted: 7) and 0 (pixel 1);
    # ox=2: 2 (pixel 2) and 1 (inserted 7); ox=3: 3 (outside 9) and 2 (pixel 2)
    assert acc.reshape(-1).tolist() == [1 + 9, 7 + 1, 2 + 7, 9 + 2]


CASES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation
    (2, 5, 4, 3, 3, 3, 4, 2, 1, 1),
    (1, 6, 6, 2, 2, 2, 3, 2, 0, 1),
    (2, 4, 5, 4, 3, 2, 2, (3, 2), (1, 0), 1),
    (1, 5, 5, 3, 3, 3, 2, 1, 1, 1),
    (1, 4, 4, 2, 3, 3, 3, 2, 2, 2),
]


def _pair(v):
    return (v, v) if np.isscalar(v) else tuple(v)


@pytest.mark.parametrize("case", CASES)
def test_exact_table_equals_the_library_transposed_convolution(case):
    N, H, W, Cin, KH, KW, Cout, s, p, d = case
    rng = np.random.default_rng(300 + H + Cin)
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, Cout)).astype(np.uint8)
    xs, ws = float(np.float32(0.021)), float(np.float32(0.013))
    q = I.Quant(xs, 101, ws, 131, None)
    _, y = oracle.conv2d_transpose(x, w, I.lut_exact(), s, p, q, dilation=d)
    xr = torch.from_numpy((x.astype(np.float64) - q.x_zp) * xs).permute(0, 3, 1, 2)
    wr = torch.from_numpy((w.astype(np.float64) - q.w_zp) * ws).permute(2, 3, 0, 1)  # [Cin, Cout, KH, KW]
    ref = torch.nn.functional.conv_transpose2d(xr, wr, stride=_pair(s), padding=_pair(p), dilation=_pair(d))
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert y.shape == ref.shape
    np.testing.assert_allclose(y.astype(np.float64), ref, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("signed", [False, True])
def test_equals_the_ordinary_layer_on_an_explicitly_spread_out_input(case, signed):
    """Spread the input out with numpy (zero-point code in between), flip the filters, and run the
    pinned ordinary oracle with stride 1 and padding dil*(K-1) - pad: the same accumulators and
    outputs for an arbitrary table and a pad code that is not the zero point."""
    N, H, W, Cin, KH, KW, Cout, s, p, d = case
    (sh, sw), (ph, pw), (dh, dw) = _pair(s), _pair(p), _pair(d)
    rng = np.random.default_rng(400 + H + Cin)
    if signed:
        x = rng.integers(-128, 128, (N, H, W, Cin)).astype(np.int8)
        w = rng.integers(-128, 128, (KH, KW, Cin, Cout)).astype(np.int8)
        lut, q = I.lut_signed_random_error(5), I.Quant(0.02, -9, 0.01, 11, 33)
    else:
        x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
        w = rng.integers(0, 256, (KH, KW, Cin, Cout)).astype(np.uint8)
        lut, q = I.lut_random(7), I.Quant(0.02, 3, 0.01, 128, 77)
    acc, y = oracle.conv2d_transpose(x, w, lut, s, p, q, dilation=d, signed=signed)
    spread = np.full((N, (H - 1) * sh + 1, (W - 1) * sw + 1, Cin), q.x_zp, dtype=x.dtype)
    spread[:, ::sh, ::sw, :] = x
    flipped = np.ascontiguousarray(w[::-1, ::-1])
    a_ref, y_ref = oracle.conv2d_ex(spread, flipped, lut, 1, (dh * (KH - 1) - ph, dw * (KW - 1) - pw), q,
                                    dilation=(dh, dw), signed=signed)
    assert np.array_equal(acc, a_ref) and np.array_equal(y, y_ref)
