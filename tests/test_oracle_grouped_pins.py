"""Pins of the grouped-convolution oracle against things other than itself (CPU only): a hand
case, the already pinned base oracle on every channel block taken alone, the depthwise oracle
(groups = Cin), and a float64 grouped library convolution of the dequantized tensors."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I


def test_hand_case_two_groups():
    """1 x 1 kernel, 4 input channels in 2 blocks, 2 output channels (one per block), exact table:
    y0 = 1*5 + 2*6 = 17 from channels 0, 1;  y1 = 3*7 + 4*8 = 53 from channels 2, 3."""
    x = np.array([1, 2, 3, 4], np.uint8).reshape(1, 1, 1, 4)
    w = np.array([[5, 7], [6, 8]], np.uint8).reshape(1, 1, 2, 2)  # [cl][co]
    acc, y = oracle.conv2d_grouped(x, w, I.lut_exact(), 1, 0, I.Quant(1.0, 0, 1.0, 0, -1), groups=2)
    assert acc.reshape(-1).tolist() == [17, 53] and y.reshape(-1).tolist() == [17.0, 53.0]
    # with zero points 1 and 2 and scale 0.5 * 0.25:  (1-1)(5-2)+(2-1)(6-2) = 4,  (3-1)(7-2)+(4-1)(8-2) = 28
    acc, y = oracle.conv2d_grouped(x, w, I.lut_exact(), 1, 0, I.Quant(0.5, 1, 0.25, 2, -1), groups=2)
    assert acc.reshape(-1).tolist() == [17, 53] and y.reshape(-1).tolist() == [0.5, 3.5]


CASES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation, groups
    (2, 9, 8, 6, 3, 3, 4, 1, 1, 1, 2),
    (1, 10, 10, 12, 3, 2, 9, 2, 2, 1, 3),
    (2, 7, 7, 8, 1, 1, 8, 1, 0, 1, 4),
    (1, 11, 9, 4, 3, 3, 6, 1, 2, 2, 2),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("signed", [False, True])
def test_every_block_is_an_ordinary_convolution_of_its_channels(case, signed):
    """Output block g equals the base (variant) oracle applied to input block g and the filters of
    output block g: pins the block assignment, the filter layout, the table addressing and the
    correction with K = KH*KW*Cin/groups, for an arbitrary (non-commutative) table."""
    N, H, W, Cin, KH, KW, Cout, s, p, d, G = case
    rng = np.random.default_rng(100 + Cin + G)
    if signed:
        x = rng.integers(-128, 128, (N, H, W, Cin)).astype(np.int8)
        w = rng.integers(-128, 128, (KH, KW, Cin // G, Cout)).astype(np.int8)
        lut = I.lut_signed_random_error(3)
        q = I.Quant(0.02, -5, 0.01, 9, 17)
    else:
        x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
        w = rng.integers(0, 256, (KH, KW, Cin // G, Cout)).astype(np.uint8)
        lut = I.lut_random(5)
        q = I.Quant(0.02, 3, 0.01, 128, 77)
    acc, y = oracle.conv2d_grouped(x, w, lut, s, p, q, groups=G, dilation=d, signed=signed)
    Cg, Cog = Cin // G, Cout // G
    for g in range(G):
        xs = np.ascontiguousarray(x[..., g * Cg:(g + 1) * Cg])
        ws = np.ascontiguousarray(w[..., g * Cog:(g + 1) * Cog])
        a_ref, y_ref = oracle.conv2d_ex(xs, ws, lut, s, p, q, dilation=d, signed=signed)
        assert np.array_equal(acc[..., g * Cog:(g + 1) * Cog], a_ref)
        assert np.array_equal(y[..., g * Cog:(g + 1) * Cog], y_ref)


def test_one_group_is_the_ordinary_layer_and_cin_groups_the_depthwise_layer():
    rng = np.random.default_rng(7)
    x = rng.integers(0, 256, (2, 8, 8, 6)).astype(np.uint8)
    lut = I.lut_random_error(2)
    q = I.Quant(0.03, 4, 0.02, 120, -1)
    w = rng.integers(0, 256, (3, 3, 6, 5)).astype(np.uint8)
    a1, y1 = oracle.conv2d_grouped(x, w, lut, 1, 1, q, groups=1)
    a0, y0 = oracle.conv2d(x, w, lut, 1, 1, q)
    assert np.array_equal(a1, a0) and np.array_equal(y1, y0)
    wd = rng.integers(0, 256, (3, 3, 6, 2)).astype(np.uint8)  # depthwise filters [KH,KW,Cin,mult]
    ad, yd = oracle.conv2d_ex(x, wd, lut, 1, 1, q, depthwise=True)
    ag, yg = oracle.conv2d_grouped(x, wd.reshape(3, 3, 1, 12), lut, 1, 1, q, groups=6)
    assert np.array_equal(ag, ad) and np.array_equal(yg, yd)


@pytest.mark.parametrize("case", CASES)
def test_exact_table_equals_the_grouped_library_convolution(case):
    """With the exact multiplier the float output is the float64 grouped convolution of the
    dequantized tensors (zero padding = the zero point's real value)."""
    N, H, W, Cin, KH, KW, Cout, s, p, d, G = case
    rng = np.random.default_rng(200 + Cin)
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin // G, Cout)).astype(np.uint8)
    xs, ws = float(np.float32(0.021)), float(np.float32(0.013))
    q = I.Quant(xs, 101, ws, 131, None)
    _, y = oracle.conv2d_grouped(x, w, I.lut_exact(), s, p, q, groups=G, dilation=d)
    xr = torch.from_numpy((x.astype(np.float64) - q.x_zp) * xs).permute(0, 3, 1, 2)
    wr = torch.from_numpy((w.astype(np.float64) - q.w_zp) * ws).permute(3, 2, 0, 1)  # [Cout, Cin/G, KH, KW]
    ref = torch.nn.functional.conv2d(xr, wr, stride=s, padding=p, dilation=d, groups=G).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(y.astype(np.float64), ref, rtol=1e-6, atol=1e-9)
