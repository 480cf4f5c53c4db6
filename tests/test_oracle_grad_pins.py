"""Pins of the backward-pass oracle against things other than itself (CPU only): hand cases,
float64 autograd of the library convolution on the dequantized tensors (also over an input
that is explicitly padded with the real value of a pad code), the bilinear identities that tie
it to the separately pinned forward oracle, and finite differences."""

import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I

import helpers as Hh

CASES = Hh.parse_cases(os.path.join(Hh.GOLDEN, "grad_cases.txt"))


def _arr(c, key, dtype):
    return np.array(c[key].split(), dtype=np.int64).astype(dtype).reshape([int(v) for v in c[key + "_shape"].split()])


@pytest.mark.parametrize("name", sorted(CASES))
def test_hand_cases(name):
    c = CASES[name]
    x, w = _arr(c, "x", np.uint8), _arr(c, "w", np.uint8)
    q = I.Quant(float(c["x_scale"]), int(c["x_zp"]), float(c["w_scale"]), int(c["w_zp"]), int(c.get("pad_code", -1)))
    s, p = int(c["stride"]), int(c["pad"])
    OH = (x.shape[1] + 2 * p - w.shape[0]) // s + 1
    OW = (x.shape[2] + 2 * p - w.shape[1]) // s + 1
    gy = np.array(c["gy"].split(), dtype=np.float32).reshape(x.shape[0], OH, OW, w.shape[3])
    r = oracle.conv2d_backward(x, w, gy, s, p, q)
    assert r["gx"].reshape(-1).tolist() == [float(v) for v in c["gx"].split()]
    assert r["gw"].reshape(-1).tolist() == [float(v) for v in c["gw"].split()]


SHAPES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation
    (2, 7, 6, 3, 3, 3, 4, 1, 1, 1),
    (1, 9, 8, 2, 3, 2, 5, 2, 1, 1),
    (2, 10, 9, 3, 3, 3, 2, (2, 3), (2, 1), (2, 1)),
    (1, 5, 5, 4, 1, 1, 6, 1, 0, 1),
    (2, 8, 8, 2, 5, 5, 3, 3, 4, 1),      # padding as large as the kernel allows, stride that skips rows
    (1, 6, 7, 2, 2, 2, 3, 2, 0, 2),
]


def _pair(v):
    return (v, v) if np.isscalar(v) else tuple(v)


def _rand(shape, seed, signed):
    N, H, W, Cin, KH, KW, Cout, s, p, d = shape
    rng = np.random.default_rng(seed)
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    x = rng.integers(lo, hi, (N, H, W, Cin)).astype(dt)
    w = rng.integers(lo, hi, (KH, KW, Cin, Cout)).astype(dt)
    # the scales are float32 parameters of the layer: take values float32 holds exactly
    q = I.Quant(float(np.float32(0.03)), int(rng.integers(lo, hi)), float(np.float32(0.007)), int(rng.integers(lo, hi)), None)
    (sh, sw), (ph, pw), (dh, dw) = _pair(s), _pair(p), _pair(d)
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    gy = rng.standard_normal((N, OH, OW, Cout)).astype(np.float32)
    return x, w, q, gy


def _autograd(x, w, q, gy, s, p, d, pad_real=0.0):
    """dL/dxr, dL/dwr of L = <gy, conv(xr, wr)> by float64 autograd of the library convolution."""
    xr = (q.x_scale * (torch.from_numpy(x.astype(np.float64)) - q.x_zp)).permute(0, 3, 1, 2).requires_grad_(True)
    wr = (q.w_scale * (torch.from_numpy(w.astype(np.float64)) - q.w_zp)).permute(3, 2, 0, 1).requires_grad_(True)
    (ph, pw) = _pair(p)
    xin = torch.nn.functional.pad(xr, (pw, pw, ph, ph), value=pad_real)
    y = torch.nn.functional.conv2d(xin, wr, stride=_pair(s), dilation=_pair(d))
    (y * torch.from_numpy(gy.astype(np.float64)).permute(0, 3, 1, 2)).sum().backward()
    return xr.grad.permute(0, 2, 3, 1).numpy(), wr.grad.permute(2, 3, 1, 0).numpy(), y.detach().permute(0, 2, 3, 1).numpy()


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_against_float64_autograd_of_the_library_convolution(shape, signed):
    x, w, q, gy = _rand(shape, 31, signed)
    s, p, d = shape[7:]
    r = oracle.conv2d_backward(x, w, gy, s, p, q, dilation=d, signed=signed)
    gx, gw, _ = _autograd(x, w, q, gy, s, p, d)
    np.testing.assert_allclose(r["gx"], gx, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(r["gw"], gw, rtol=1e-11, atol=1e-11)
    # the sums of absolute values bound the sums, and are what they say
    assert np.all(np.abs(r["gx"]) <= r["gx_abs"] * (1 + 1e-12) + 1e-300)
    assert np.all(np.abs(r["gw"]) <= r["gw_abs"] * (1 + 1e-12) + 1e-300)


def test_pad_code_that_is_not_the_zero_point_enters_the_filter_gradient():
    shape = (2, 6, 5, 3, 3, 3, 4, 1, 2, 1)
    x, w, q, gy = _rand(shape, 33, False)
    q = I.Quant(q.x_scale, 100, q.w_scale, 77, 13)  # padded taps carry 0.03 * (13 - 100)
    r = oracle.conv2d_backward(x, w, gy, 1, 2, q)
    gx, gw, _ = _autograd(x, w, q, gy, 1, 2, 1, pad_real=q.x_scale * (13 - 100))
    np.testing.assert_allclose(r["gx"], gx, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(r["gw"], gw, rtol=1e-11, atol=1e-11)
    gx0, gw0, _ = _autograd(x, w, q, gy, 1, 2, 1, pad_real=0.0)
    assert np.allclose(gx0, gx) and not np.allclose(gw0, gw)  # the pad value changes gw only


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_bilinear_identities_tie_the_backward_to_the_forward_oracle(shape):
    """y is linear in xr and in wr, so <gx, xr> = <gw, wr> = <gy, y> (zero padding); y is taken
    from the forward oracle with the exact table, which is pinned separately."""
    x, w, q, gy = _rand(shape, 35, False)
    s, p, d = shape[7:]
    r = oracle.conv2d_backward(x, w, gy, s, p, q, dilation=d)
    _, y = oracle.conv2d_ex(x, w, I.lut_exact(), s, p, q, dilation=d)
    L = float((gy.astype(np.float64) * y.astype(np.float64)).sum())
    xr = q.x_scale * (x.astype(np.float64) - q.x_zp)
    wr = q.w_scale * (w.astype(np.float64) - q.w_zp)
    scale = float(np.abs(gy.astype(np.float64) * y.astype(np.float64)).sum())
    assert abs(float((r["gx"] * xr).sum()) - L) <= 1e-5 * scale  # y is a float32 tensor
    assert abs(float((r["gw"] * wr).sum()) - L) <= 1e-5 * scale


def test_finite_differences_on_a_tiny_layer():
    """Central differences of L(xr, wr) = <gy, conv(xr, wr)> computed by explicit loops here."""
    rng = np.random.default_rng(37)
    N, H, W, Cin, KH, KW, Cout, s, p = 1, 4, 3, 2, 2, 2, 2, 1, 1
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, Cout)).astype(np.uint8)
    q = I.Quant(0.5, 100, 0.25, 90, None)
    OH, OW = H + 2 * p - KH + 1, W + 2 * p - KW + 1
    gy = rng.standard_normal((N, OH, OW, Cout)).astype(np.float32)

    def loss(xr, wr):
        tot = 0.0
        for oy in range(OH):
            for ox in range(OW):
                for co in range(Cout):
                    acc = 0.0
                    for ky in range(KH):
                        for kx in range(KW):
                            iy, ix = oy - p + ky, ox - p + kx
                            if 0 <= iy < H and 0 <= ix < W:
                                acc += float((xr[0, iy, ix, :] * wr[ky, kx, :, co]).sum())
                    tot += acc * float(gy[0, oy, ox, co])
        return tot

    xr = q.x_scale * (x.astype(np.float64) - q.x_zp)
    wr = q.w_scale * (w.astype(np.float64) - q.w_zp)
    r = oracle.conv2d_backward(x, w, gy, s, p, q)
    for idx in [(0, 0, 0, 0), (0, 3, 2, 1), (0, 1, 1, 0)]:
        e = np.zeros_like(xr); e[idx] = 1e-3
        fd = (loss(xr + e, wr) - loss(xr - e, wr)) / 2e-3
        assert abs(fd - r["gx"][idx]) <= 1e-7 * max(1.0, abs(fd))
    for idx in [(0, 0, 0, 0), (1, 1, 1, 1), (0, 1, 1, 0)]:
        e = np.zeros_like(wr); e[idx] = 1e-3
        fd = (loss(xr, wr + e) - loss(xr, wr - e)) / 2e-3
        assert abs(fd - r["gw"][idx]) <= 1e-7 * max(1.0, abs(fd))
