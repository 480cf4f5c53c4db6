"""Pins of the operator-variant oracle (dilation, signed codes, depthwise) against things other
than itself (CPU only): hand cases, the already pinned base oracle on the special cases that
reduce to it, numpy gathers over explicitly padded arrays, float64 library convolutions."""

import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I

import helpers as Hh

CASES = Hh.parse_cases(os.path.join(Hh.GOLDEN, "hand_cases.txt"))


def _arr(c, key, dtype):
    return np.array(c[key].split(), dtype=np.int64).astype(dtype).reshape([int(v) for v in c[key + "_shape"].split()])


def test_hand_signed_case():
    c = CASES["case_S1"]
    q = I.Quant(float(c["x_scale"]), int(c["x_zp"]), float(c["w_scale"]), int(c["w_zp"]), None)
    acc, y = oracle.conv2d_ex(_arr(c, "x", np.int8), _arr(c, "w", np.int8), I.lut_signed_exact(), 1, 0, q, signed=True)
    assert acc.reshape(-1).tolist() == [int(c["acc"])] and y.reshape(-1).tolist() == [float(c["y"])]


def test_hand_dilation_case():
    c = CASES["case_D1"]
    acc, y = oracle.conv2d_ex(_arr(c, "x", np.uint8), _arr(c, "w", np.uint8), I.lut_exact(), 1, 0,
                              I.Quant(1.0, 0, 1.0, 0, -1), dilation=2)
    assert acc.shape == (1, 1, 1, 1) and int(acc.reshape(-1)[0]) == int(c["acc"]) and float(y.reshape(-1)[0]) == float(c["y"])


def test_hand_depthwise_case():
    c = CASES["case_W1"]
    acc, y = oracle.conv2d_ex(_arr(c, "x", np.uint8), _arr(c, "w", np.uint8), I.lut_exact(), 1, 0,
                              I.Quant(1.0, 0, 1.0, 0, -1), depthwise=True)
    assert acc.reshape(-1).tolist() == [int(v) for v in c["acc"].split()]
    assert y.reshape(-1).tolist() == [float(v) for v in c["y"].split()]


SHAPES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation
    (1, 12, 12, 4, 3, 3, 5, 1, 2, 2),
    (2, 11, 9, 3, 3, 2, 4, 2, 3, 3),
    (1, 9, 9, 2, 2, 2, 3, 1, 0, (2, 3)),
    (2, 8, 8, 5, 3, 3, 6, (2, 1), (1, 4), (1, 2)),
]


def _pair(v):
    return (v, v) if np.isscalar(v) else tuple(v)


def _gather(x, w, lut_fn, s, p, d, pad_code):
    """Definition by explicit padding and fancy indexing: returns sum over taps of lut_fn(a, b)
    plus Sp, Sf, for ordinary convolutions.  x, w integer arrays of any signedness."""
    (sh, sw), (ph, pw), (dh, dw) = _pair(s), _pair(p), _pair(d)
    N, H, W, C = x.shape
    KH, KW, _, Co = w.shape
    xp = np.full((N, H + 2 * ph, W + 2 * pw, C), pad_code, dtype=np.int64)
    xp[:, ph:ph + H, pw:pw + W, :] = x
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    acc = np.zeros((N, OH, OW, Co), np.int64)
    Sp = np.zeros((N, OH, OW), np.int64)
    for ky in range(KH):
        for kx in range(KW):
            a = xp[:, ky * dh:ky * dh + (OH - 1) * sh + 1:sh, kx * dw:kx * dw + (OW - 1) * sw + 1:sw, :]  # N,OH,OW,C
            b = w[ky, kx].astype(np.int64)  # C,Co
            acc += lut_fn(a[..., :, None], b[None, None, None, :, :]).sum(axis=3)
            Sp += a.sum(axis=3)
    Sf = w.astype(np.int64).sum(axis=(0, 1, 2))
    return acc, Sp, Sf


def _q(rng, signed=False):
    lo, hi = (-128, 128) if signed else (0, 256)
    return I.Quant(0.03, int(rng.integers(lo, hi)), 0.007, int(rng.integers(lo, hi)), None)


def test_dilation_one_is_the_base_oracle():
    rng = np.random.default_rng(1)
    x = rng.integers(0, 256, (2, 9, 7, 5)).astype(np.uint8)
    w = rng.integers(0, 256, (3, 3, 5, 6)).astype(np.uint8)
    lut = I.lut_random(3)
    q = I.Quant(0.02, 31, 0.005, 200, 77)
    a0, y0 = oracle.conv2d(x, w, lut, 2, 1, q)
    a1, y1 = oracle.conv2d_ex(x, w, lut, 2, 1, q)
    np.testing.assert_array_equal(a0, a1)
    np.testing.assert_array_equal(y0, y1)


@pytest.mark.parametrize("shape", SHAPES)
def test_dilated_convolution_against_gather_and_library(shape):
    N, H, W, Cin, KH, KW, Cout, s, p, d = shape
    rng = np.random.default_rng(2)
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, Cout)).astype(np.uint8)
    q = _q(rng)
    lut = I.lut_random(4)
    acc, y = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d)
    ref, Sp, Sf = _gather(x, w, lambda a, b: lut.reshape(256, 256).astype(np.int64)[a, b], s, p, d, q.x_zp)
    np.testing.assert_array_equal(acc, ref)
    K = KH * KW * Cin
    corr = ref - q.w_zp * Sp[..., None] - q.x_zp * Sf + K * q.x_zp * q.w_zp
    assert Hh.float_ok(y, np.float64(q.x_scale) * np.float64(q.w_scale) * corr)
    # exact table: the library's dilated float64 convolution of the dequantized tensors
    acc, y = oracle.conv2d_ex(x, w, I.lut_exact(), s, p, q, dilation=d)
    xr = q.x_scale * (torch.from_numpy(x.astype(np.float64)) - q.x_zp)
    wr = q.w_scale * (torch.from_numpy(w.astype(np.float64)) - q.w_zp)
    lib = torch.nn.functional.conv2d(xr.permute(0, 3, 1, 2), wr.permute(3, 2, 0, 1), stride=_pair(s), padding=_pair(p),
                                     dilation=_pair(d)).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y, lib, rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("mult", [1, 3])
@pytest.mark.parametrize("d", [1, 2])
def test_depthwise_is_one_single_channel_convolution_per_output_channel(mult, d):
    rng = np.random.default_rng(5)
    N, H, W, Cin, KH, KW, s, p = 2, 8, 7, 4, 3, 3, 2, 1
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, mult)).astype(np.uint8)
    q = I.Quant(0.02, 17, 0.004, 140, 9)
    lut = I.lut_random(6)
    acc, y = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d, depthwise=True)
    assert acc.shape[-1] == Cin * mult
    for ci in range(Cin):
        for m in range(mult):
            xs = np.ascontiguousarray(x[..., ci:ci + 1])
            wsl = np.ascontiguousarray(w[:, :, ci:ci + 1, m:m + 1])
            if d == 1:
                a1, y1 = oracle.conv2d(xs, wsl, lut, s, p, q)  # the separately pinned base oracle
            else:
                a1, _, _ = _gather(xs, wsl, lambda a, b: lut.reshape(256, 256).astype(np.int64)[a, b], s, p, d, q.pad_code)
                y1 = None
            np.testing.assert_array_equal(acc[..., ci * mult + m], a1[..., 0])
            if y1 is not None:
                np.testing.assert_array_equal(y[..., ci * mult + m], y1[..., 0])


def test_depthwise_exact_table_equals_grouped_library_convolution():
    rng = np.random.default_rng(7)
    N, H, W, Cin, mult = 2, 9, 9, 6, 2
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (3, 3, Cin, mult)).astype(np.uint8)
    q = _q(rng)
    acc, y = oracle.conv2d_ex(x, w, I.lut_exact(), 1, 1, q, depthwise=True)
    xr = q.x_scale * (torch.from_numpy(x.astype(np.float64)) - q.x_zp)
    wr = q.w_scale * (torch.from_numpy(w.astype(np.float64)) - q.w_zp)
    # torch wants [Cin*mult, 1, KH, KW] with output channel ci*mult + m
    wt = wr.permute(2, 3, 0, 1).reshape(Cin * mult, 1, 3, 3)
    lib = torch.nn.functional.conv2d(xr.permute(0, 3, 1, 2), wt, padding=1, groups=Cin).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y, lib, rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("shape", SHAPES)
def test_signed_exact_table_is_integer_convolution(shape):
    N, H, W, Cin, KH, KW, Cout, s, p, d = shape
    rng = np.random.default_rng(8)
    x = rng.integers(-128, 128, (N, H, W, Cin)).astype(np.int8)
    w = rng.integers(-128, 128, (KH, KW, Cin, Cout)).astype(np.int8)
    q = _q(rng, signed=True)
    acc, y = oracle.conv2d_ex(x, w, I.lut_signed_exact(), s, p, q, dilation=d, signed=True)
    ref, Sp, Sf = _gather(x.astype(np.int64), w.astype(np.int64), lambda a, b: a * b, s, p, d, q.x_zp)
    np.testing.assert_array_equal(acc, ref)
    xr = q.x_scale * (torch.from_numpy(x.astype(np.float64)) - q.x_zp)
    wr = q.w_scale * (torch.from_numpy(w.astype(np.float64)) - q.w_zp)
    lib = torch.nn.functional.conv2d(xr.permute(0, 3, 1, 2), wr.permute(3, 2, 0, 1), stride=_pair(s), padding=_pair(p),
                                     dilation=_pair(d)).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y, lib, rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("table", ["error", "random"])
def test_signed_layer_is_the_unsigned_layer_in_offset_binary(table):
    """Adding 128 to every code and zero point and re-addressing / re-biasing the table turns a
    signed layer into an unsigned one (handled by the separately pinned base oracle):
    acc_signed = acc_unsigned - 32768*K.  A non-symmetric table also pins the
    order of the two stitched patterns."""
    rng = np.random.default_rng(9)
    x = rng.integers(-128, 128, (2, 7, 6, 5)).astype(np.int8)
    w = rng.integers(-128, 128, (3, 3, 5, 4)).astype(np.int8)
    lut_s = I.lut_signed_random_error(3) if table == "error" else I.lut_signed_random(4)
    q = I.Quant(0.02, -5, 0.01, 90, 33)
    acc, y = oracle.conv2d_ex(x, w, lut_s, 1, 1, q, signed=True)
    v = np.arange(256) - 128                       # value of offset-binary code c' is c' - 128
    lut_u = (lut_s.reshape(256, 256).astype(np.int64)[np.ix_(v & 255, v & 255)] + 32768).astype(np.uint16)
    xu = (x.astype(np.int64) + 128).astype(np.uint8)
    wu = (w.astype(np.int64) + 128).astype(np.uint8)
    qu = I.Quant(q.x_scale, q.x_zp + 128, q.w_scale, q.w_zp + 128, q.pad_code + 128)
    acc_u, y_u = oracle.conv2d(xu, wu, lut_u, 1, 1, qu)
    K = 3 * 3 * 5
    np.testing.assert_array_equal(acc.astype(np.int64), acc_u.astype(np.int64) - 32768 * K)
    # (the float outputs of the two layers differ: the correction terms of Eq. (3) are taken on
    # the signed codes and zero points; the signed correction is pinned by the exact-table test)
    del y, y_u


def test_signed_layer_float_output_with_a_pad_code_that_is_not_the_zero_point():
    """The float output of a signed layer whose padded taps carry a code other than the zero
    point, pinned twice without the oracle's own correction line: (a) an arbitrary signed table
    against acc, Sp, Sf gathered in numpy and put through the expansion of Eq. (3) here;
    (b) the exact table against a float64 library convolution of the dequantized tensors over an
    input that is explicitly padded with the real value of the pad code, alpha1*(pad - beta1)."""
    rng = np.random.default_rng(21)
    N, H, W, Cin, KH, KW, Cout, s, p, d = 2, 7, 6, 5, 3, 3, 4, 1, 2, 1
    x = rng.integers(-128, 128, (N, H, W, Cin)).astype(np.int8)
    w = rng.integers(-128, 128, (KH, KW, Cin, Cout)).astype(np.int8)
    q = I.Quant(0.02, -9, 0.01, 41, 77)  # pad code 77, zero point -9
    K = KH * KW * Cin
    lut = I.lut_signed_random(5)
    acc, y = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d, signed=True)
    tab = lut.reshape(256, 256).astype(np.int64)
    ref, Sp, Sf = _gather(x.astype(np.int64), w.astype(np.int64), lambda a, b: tab[a & 255, b & 255], s, p, d, q.pad_code)
    np.testing.assert_array_equal(acc, ref)
    corr = ref - q.w_zp * Sp[..., None] - q.x_zp * Sf + K * q.x_zp * q.w_zp
    assert Hh.float_ok(y, np.float64(q.x_scale) * np.float64(q.w_scale) * corr)
    # (b): padded taps are real numbers here, not zeros
    _, y_exact = oracle.conv2d_ex(x, w, I.lut_signed_exact(), s, p, q, dilation=d, signed=True)
    xr = q.x_scale * (torch.from_numpy(x.astype(np.float64)) - q.x_zp)
    wr = q.w_scale * (torch.from_numpy(w.astype(np.float64)) - q.w_zp)
    pad_real = q.x_scale * (q.pad_code - q.x_zp)
    xpad = torch.nn.functional.pad(xr.permute(0, 3, 1, 2), (p, p, p, p), value=pad_real)
    lib = torch.nn.functional.conv2d(xpad, wr.permute(3, 2, 0, 1), stride=s).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y_exact, lib, rtol=1e-5, atol=1e-4)
    assert not Hh.float_ok(y_exact, torch.nn.functional.conv2d(xr.permute(0, 3, 1, 2), wr.permute(3, 2, 0, 1), stride=s,
                                                                padding=p).permute(0, 2, 3, 1).numpy(), rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("mult", [1, 2])
def test_depthwise_with_dilation_float_output(mult):
    """Depthwise and dilated at once: accumulators and float outputs per output channel against
    a numpy gather and the expansion of Eq. (3) written out here (K = KH*KW), and the exact
    table against the library's grouped, dilated float64 convolution."""
    rng = np.random.default_rng(23)
    N, H, W, Cin, KH, KW, s, p, d = 2, 10, 9, 3, 3, 3, 1, 2, 2
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, mult)).astype(np.uint8)
    q = I.Quant(0.02, 17, 0.004, 140, 9)  # pad code 9 is not the zero point
    lut = I.lut_random(8)
    tab = lut.reshape(256, 256).astype(np.int64)
    acc, y = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d, depthwise=True)
    K = KH * KW
    for ci in range(Cin):
        for m in range(mult):
            a1, Sp, Sf = _gather(x[..., ci:ci + 1].astype(np.int64), w[:, :, ci:ci + 1, m:m + 1].astype(np.int64),
                                 lambda a, b: tab[a, b], s, p, d, q.pad_code)
            co = ci * mult + m
            np.testing.assert_array_equal(acc[..., co], a1[..., 0])
            corr = a1[..., 0] - q.w_zp * Sp - q.x_zp * Sf[0] + K * q.x_zp * q.w_zp
            assert Hh.float_ok(y[..., co], np.float64(q.x_scale) * np.float64(q.w_scale) * corr)
    qz = I.Quant(0.02, 17, 0.004, 140, None)  # padded taps are real zeros
    _, y_exact = oracle.conv2d_ex(x, w, I.lut_exact(), s, p, qz, dilation=d, depthwise=True)
    xr = qz.x_scale * (torch.from_numpy(x.astype(np.float64)) - qz.x_zp)
    wr = qz.w_scale * (torch.from_numpy(w.astype(np.float64)) - qz.w_zp)
    wt = wr.permute(2, 3, 0, 1).reshape(Cin * mult, 1, KH, KW)
    lib = torch.nn.functional.conv2d(xr.permute(0, 3, 1, 2), wt, padding=p, dilation=d, groups=Cin).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y_exact, lib, rtol=1e-5, atol=1e-4)
