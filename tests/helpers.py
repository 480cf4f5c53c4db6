"""Helpers for the tests: golden-file parser and an independent numpy formulation of the
layer (gather over an explicitly padded array) used to pin the C oracle."""

import os

import numpy as np

from paper_2002_09481_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def parse_cases(path):
    cases, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("["):
                cur = cases.setdefault(line.strip("[]"), {})
                continue
            k, v = [s.strip() for s in line.split("=", 1)]
            cur[k] = v
    return cases


def named_lut(spec):
    parts = spec.split()
    if parts[0] == "exact":
        return I.lut_exact()
    if parts[0] == "truncated":
        return I.lut_truncated(int(parts[1]))
    if parts[0] == "first":
        return I.lut_first_operand()
    if parts[0] == "second":
        return I.lut_second_operand()
    raise ValueError(spec)


def case_operands(c):
    x = np.array(c["x"].split(), dtype=np.int64).astype(np.uint8).reshape([int(v) for v in c["x_shape"].split()])
    w = np.array(c["w"].split(), dtype=np.int64).astype(np.uint8).reshape([int(v) for v in c["w_shape"].split()])
    q = I.Quant(float(c["x_scale"]), int(c["x_zp"]), float(c["w_scale"]), int(c["w_zp"]), int(c["pad_code"]))
    acc = np.array(c["acc"].split(), dtype=np.int64)
    y = np.array(c["y"].split(), dtype=np.float64)
    return x, w, named_lut(c["lut"]), int(c["stride"]), int(c["pad"]), q, acc, y


def patches(x, KH, KW, stride, pad, pad_code):
    """[N,OH,OW,KH,KW,Cin] int64 view of the explicitly padded input."""
    N, H, W, C = x.shape
    xp = np.full((N, H + 2 * pad, W + 2 * pad, C), pad_code, dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    win = np.lib.stride_tricks.sliding_window_view(xp, (KH, KW), axis=(1, 2))  # N,OH',OW',C,KH,KW
    win = win[:, ::stride, ::stride]
    return np.ascontiguousarray(np.transpose(win, (0, 1, 2, 4, 5, 3)))


def numpy_lut_conv(x, w, lut, stride, pad, pad_code):
    """acc[n,oy,ox,co] = sum over taps of lut2d[patch, w] by fancy indexing (small inputs only)."""
    KH, KW, Cin, Cout = w.shape
    p = patches(x, KH, KW, stride, pad, pad_code)  # N,OH,OW,KH,KW,Cin
    lut2d = np.asarray(lut).reshape(256, 256).astype(np.int64)
    g = lut2d[p[..., None], w.astype(np.int64)[None, None, None]]  # N,OH,OW,KH,KW,Cin,Cout
    return g.sum(axis=(3, 4, 5))


def numpy_int_conv(x, w, stride, pad, pad_code):
    """Plain integer convolution (exact products) by einsum on the padded patches."""
    KH, KW, Cin, Cout = w.shape
    p = patches(x, KH, KW, stride, pad, pad_code)
    return np.einsum("nyxhwc,hwco->nyxo", p, w.astype(np.int64))


def float_ok(y, ref, rtol=1e-5, atol=1e-6):
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.all(np.abs(y - ref) <= rtol * np.abs(ref) + atol)
