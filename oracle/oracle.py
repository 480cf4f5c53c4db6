"""ctypes loader for the C oracle.  Test infrastructure: imported only by tests/, the smoke
check and the benchmark's cpu_baseline leg.  Takes and returns numpy arrays on the host."""

from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


class _Quant(ctypes.Structure):
    _fields_ = [
        ("x_scale", ctypes.c_float),
        ("x_zp", ctypes.c_int32),
        ("w_scale", ctypes.c_float),
        ("w_zp", ctypes.c_int32),
        ("pad_code", ctypes.c_int32),
    ]


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        _lib.ax_oracle_conv2d.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, vp, vp, vp]
        _lib.ax_oracle_conv2d_sample.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, vp, vp, ci, vp, vp]
        _lib.ax_oracle_dense.argtypes = [vp, ci, ci, vp, ci, vp, vp, vp, vp]
        i64, cf = ctypes.c_int64, ctypes.c_float
        _lib.ax_oracle_range_f32.argtypes = [vp, i64, ci, vp]
        _lib.ax_oracle_coeffs.argtypes = [vp, ci, vp, vp]
        _lib.ax_oracle_quantize_f32.argtypes = [vp, i64, ci, cf, ctypes.c_int32, ci, vp]
        _lib.ax_oracle_conv2d_f32.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, vp, vp, ci, ci,
                                              vp, vp, vp, vp, vp]
        _lib.ax_oracle_conv2d_ex.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci,
                                             cf, ci, cf, ci, ci, vp, vp]
        _lib.ax_oracle_conv2d_ex.restype = ci
        _lib.ax_oracle_conv2d_grouped.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci,
                                             cf, ci, cf, ci, ci, vp, vp]
        _lib.ax_oracle_conv2d_grouped.restype = ci
        _lib.ax_oracle_conv2d_transpose.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci,
                                                    cf, ci, cf, ci, ci, vp, vp]
        _lib.ax_oracle_conv2d_transpose.restype = ci
        _lib.ax_oracle_conv2d_f32_ex.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci,
                                                 vp, vp, ci, ci, vp, vp, vp, vp, vp]
        _lib.ax_oracle_conv2d_f32_ex.restype = ci
        _lib.ax_oracle_conv2d_backward.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, ci,
                                                   cf, ci, cf, ci, ci, vp, vp, vp, vp, vp]
        _lib.ax_oracle_conv2d_backward.restype = ci
        for f in (_lib.ax_oracle_conv2d, _lib.ax_oracle_conv2d_sample, _lib.ax_oracle_dense, _lib.ax_oracle_threads,
                  _lib.ax_oracle_range_f32, _lib.ax_oracle_coeffs, _lib.ax_oracle_quantize_f32,
                  _lib.ax_oracle_conv2d_f32):
            f.restype = ci
    return _lib


def _q(q) -> _Quant:
    return _Quant(float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), int(q.pad_code))


def _chk(a, dtype, ndim):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype or a.ndim != ndim:
        raise TypeError("expected %s array with %d dims, got %s %s" % (dtype, ndim, a.dtype, a.shape))
    return a


def _lut(lut):
    lut = _chk(np.asarray(lut).reshape(-1), np.uint16, 1)
    if lut.size != 65536:
        raise ValueError("table must have 65536 entries")
    return lut


def out_hw(H, W, KH, KW, stride, pad):
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    return (H + 2 * ph - KH) // sh + 1, (W + 2 * pw - KW) // sw + 1, sh, sw, ph, pw


def conv2d(x, w, lut, stride, pad, q):
    x, w, lut = _chk(x, np.uint8, 4), _chk(w, np.uint8, 4), _lut(lut)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH, OW, sh, sw, ph, pw = out_hw(H, W, KH, KW, stride, pad)
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    qs = _q(q)
    rc = lib().ax_oracle_conv2d(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                sh, sw, ph, pw, ctypes.addressof(qs), acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d failed: %d" % rc)
    return acc, y


def conv2d_sample(x, w, lut, stride, pad, q, flat_index):
    x, w, lut = _chk(x, np.uint8, 4), _chk(w, np.uint8, 4), _lut(lut)
    idx = _chk(np.asarray(flat_index, dtype=np.int64), np.int64, 1)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH, OW, sh, sw, ph, pw = out_hw(H, W, KH, KW, stride, pad)
    acc = np.empty(idx.size, np.int32)
    y = np.empty(idx.size, np.float32)
    qs = _q(q)
    rc = lib().ax_oracle_conv2d_sample(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                       sh, sw, ph, pw, ctypes.addressof(qs), idx.ctypes.data, idx.size,
                                       acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_sample failed: %d" % rc)
    return acc, y


def dense(x, w, lut, q):
    x, w, lut = _chk(x, np.uint8, 2), _chk(w, np.uint8, 2), _lut(lut)
    M, K = x.shape
    K2, N = w.shape
    if K2 != K:
        raise ValueError("inner dimension mismatch")
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.float32)
    qs = _q(q)
    rc = lib().ax_oracle_dense(x.ctypes.data, M, K, w.ctypes.data, N, lut.ctypes.data, ctypes.addressof(qs),
                               acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_dense failed: %d" % rc)
    return acc, y


def conv2d_ex(x, w, lut, stride, pad, q, dilation=1, depthwise=False, signed=False):
    """Operator variants.  signed: x, w int8 and lut int16 (addressed by the two's-complement
    patterns); depthwise: w is [KH,KW,Cin,mult].  q.pad_code None selects the zero point."""
    cdt = np.int8 if signed else np.uint8
    ldt = np.int16 if signed else np.uint16
    x, w = _chk(x, cdt, 4), _chk(w, cdt, 4)
    lut = _chk(np.asarray(lut).reshape(-1), ldt, 1)
    if lut.size != 65536:
        raise ValueError("table must have 65536 entries")
    N, H, W, Cin = x.shape
    KH, KW, Cin2, last = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    Cout = Cin * last if depthwise else last
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dilation, dilation) if np.isscalar(dilation) else dilation
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    pad_code = q.pad_code
    if pad_code is None or (not signed and pad_code < 0):
        pad_code = q.x_zp
    rc = lib().ax_oracle_conv2d_ex(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                   sh, sw, ph, pw, dh, dw, int(bool(depthwise)), int(bool(signed)),
                                   float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), int(pad_code),
                                   acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_ex failed: %d" % rc)
    return acc, y


def conv2d_grouped(x, w, lut, stride, pad, q, groups, dilation=1, signed=False):
    """Grouped convolution: w is [KH,KW,Cin/groups,Cout]."""
    cdt = np.int8 if signed else np.uint8
    ldt = np.int16 if signed else np.uint16
    x, w = _chk(x, cdt, 4), _chk(w, cdt, 4)
    lut = _chk(np.asarray(lut).reshape(-1), ldt, 1)
    if lut.size != 65536:
        raise ValueError("table must have 65536 entries")
    N, H, W, Cin = x.shape
    KH, KW, Cg, Cout = w.shape
    if groups < 1 or Cin % groups or Cout % groups or Cg * groups != Cin:
        raise ValueError("channel counts do not fit the groups")
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dilation, dilation) if np.isscalar(dilation) else dilation
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    pad_code = q.pad_code
    if pad_code is None or (not signed and pad_code < 0):
        pad_code = q.x_zp
    rc = lib().ax_oracle_conv2d_grouped(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                        sh, sw, ph, pw, dh, dw, int(groups), int(bool(signed)),
                                        float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), int(pad_code),
                                        acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_grouped failed: %d" % rc)
    return acc, y


def conv2d_transpose(x, w, lut, stride, pad, q, dilation=1, signed=False):
    """Transposed convolution by zero insertion: w is [KH,KW,Cin,Cout]."""
    cdt = np.int8 if signed else np.uint8
    ldt = np.int16 if signed else np.uint16
    x, w = _chk(x, cdt, 4), _chk(w, cdt, 4)
    lut = _chk(np.asarray(lut).reshape(-1), ldt, 1)
    if lut.size != 65536:
        raise ValueError("table must have 65536 entries")
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dilation, dilation) if np.isscalar(dilation) else dilation
    OH = (H - 1) * sh + 1 + dh * (KH - 1) - 2 * ph
    OW = (W - 1) * sw + 1 + dw * (KW - 1) - 2 * pw
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    pad_code = q.pad_code
    if pad_code is None or (not signed and pad_code < 0):
        pad_code = q.x_zp
    rc = lib().ax_oracle_conv2d_transpose(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                          sh, sw, ph, pw, dh, dw, int(bool(signed)), float(q.x_scale), int(q.x_zp),
                                          float(q.w_scale), int(q.w_zp), int(pad_code), acc.ctypes.data, y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_transpose failed: %d" % rc)
    return acc, y


def range_f32(x, relu=False):
    """(min, max) of a float32 tensor as a float32 array of two."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = np.empty(2, np.float32)
    rc = lib().ax_oracle_range_f32(x.ctypes.data, x.size, int(bool(relu)), out.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_range_f32 failed: %d" % rc)
    return out


def coeffs(rng, round_mode=0):
    """(alpha, beta) for a range of two float32 values."""
    rng = _chk(np.asarray(rng, dtype=np.float32), np.float32, 1)
    a = ctypes.c_float()
    b = ctypes.c_int32()
    rc = lib().ax_oracle_coeffs(rng.ctypes.data, int(round_mode), ctypes.addressof(a), ctypes.addressof(b))
    if rc:
        raise RuntimeError("ax_oracle_coeffs failed: %d" % rc)
    return float(a.value), int(b.value)


def quantize_f32(x, alpha, beta, relu=False, round_mode=0):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint8)
    rc = lib().ax_oracle_quantize_f32(x.ctypes.data, x.size, int(bool(relu)), float(alpha), int(beta),
                                      int(round_mode), out.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_quantize_f32 failed: %d" % rc)
    return out


def conv2d_f32(x, w, lut, stride, pad, x_range, w_range, relu=False, round_mode=0):
    """Float layer.  Returns dict(acc, y, xq, wq, x_scale, x_zp, w_scale, w_zp)."""
    x, w, lut = _chk(x, np.float32, 4), _chk(w, np.float32, 4), _lut(lut)
    xr = _chk(np.asarray(x_range, dtype=np.float32), np.float32, 1)
    wr = _chk(np.asarray(w_range, dtype=np.float32), np.float32, 1)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH, OW, sh, sw, ph, pw = out_hw(H, W, KH, KW, stride, pad)
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    xq = np.empty(x.shape, np.uint8)
    wq = np.empty(w.shape, np.uint8)
    qs = _Quant()
    rc = lib().ax_oracle_conv2d_f32(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                    sh, sw, ph, pw, xr.ctypes.data, wr.ctypes.data, int(bool(relu)), int(round_mode),
                                    xq.ctypes.data, wq.ctypes.data, ctypes.addressof(qs), acc.ctypes.data,
                                    y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_f32 failed: %d" % rc)
    return dict(acc=acc, y=y, xq=xq, wq=wq, x_scale=float(qs.x_scale), x_zp=int(qs.x_zp),
                w_scale=float(qs.w_scale), w_zp=int(qs.w_zp))


def conv2d_f32_ex(x, w, lut, stride, pad, x_range, w_range, relu=False, round_mode=0, dilation=1, depthwise=False,
                  signed=False):
    """Float layer with dilation / signed codes / depthwise filters ([KH,KW,Cin,mult]).
    Returns dict(acc, y, xq, wq, x_scale, x_zp, w_scale, w_zp); codes are int8 when signed."""
    x, w = _chk(x, np.float32, 4), _chk(w, np.float32, 4)
    lut = _chk(np.asarray(lut).reshape(-1), np.int16 if signed else np.uint16, 1)
    if lut.size != 65536:
        raise ValueError("table must have 65536 entries")
    xr = _chk(np.asarray(x_range, dtype=np.float32), np.float32, 1)
    wr = _chk(np.asarray(w_range, dtype=np.float32), np.float32, 1)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, last = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    Cout = Cin * last if depthwise else last
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dilation, dilation) if np.isscalar(dilation) else dilation
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    if OH <= 0 or OW <= 0:
        raise ValueError("empty output")
    acc = np.empty((N, OH, OW, Cout), np.int32)
    y = np.empty((N, OH, OW, Cout), np.float32)
    xq = np.empty(x.shape, np.uint8)
    wq = np.empty(w.shape, np.uint8)
    qs = _Quant()
    rc = lib().ax_oracle_conv2d_f32_ex(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, lut.ctypes.data,
                                       sh, sw, ph, pw, dh, dw, int(bool(depthwise)), int(bool(signed)),
                                       xr.ctypes.data, wr.ctypes.data, int(bool(relu)), int(round_mode),
                                       xq.ctypes.data, wq.ctypes.data, ctypes.addressof(qs), acc.ctypes.data,
                                       y.ctypes.data)
    if rc:
        raise RuntimeError("ax_oracle_conv2d_f32_ex failed: %d" % rc)
    if signed:
        xq, wq = xq.view(np.int8), wq.view(np.int8)
    return dict(acc=acc, y=y, xq=xq, wq=wq, x_scale=float(qs.x_scale), x_zp=int(qs.x_zp),
                w_scale=float(qs.w_scale), w_zp=int(qs.w_zp))


def conv2d_backward(x, w, gy, stride, pad, q, dilation=1, signed=False, want_gx=True, want_gw=True):
    """Backward pass of the layer (straight-through: gradients of the exact convolution of the
    dequantized tensors).  x, w: codes; gy: float32 [N,OH,OW,Cout].  Returns a dict with float64
    arrays gx [N,H,W,Cin], gw [KH,KW,Cin,Cout] and gx_abs, gw_abs (sums of the absolute values of
    the terms of every sum); an entry is None when not wanted."""
    cdt = np.int8 if signed else np.uint8
    x, w = _chk(x, cdt, 4), _chk(w, cdt, 4)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    dh, dw = (dilation, dilation) if np.isscalar(dilation) else dilation
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    gy = _chk(gy, np.float32, 4)
    if gy.shape != (N, OH, OW, Cout):
        raise ValueError("gy must be [N,OH,OW,Cout]")
    pad_code = q.pad_code
    if pad_code is None or (not signed and pad_code < 0):
        pad_code = q.x_zp
    out = dict(gx=None, gx_abs=None, gw=None, gw_abs=None)
    if want_gx:
        out["gx"], out["gx_abs"] = np.empty(x.shape, np.float64), np.empty(x.shape, np.float64)
    if want_gw:
        out["gw"], out["gw_abs"] = np.empty(w.shape, np.float64), np.empty(w.shape, np.float64)
    p = lambda a: None if a is None else a.ctypes.data
    rc = lib().ax_oracle_conv2d_backward(x.ctypes.data, N, H, W, Cin, w.ctypes.data, KH, KW, Cout, sh, sw, ph, pw,
                                         dh, dw, int(bool(signed)), float(q.x_scale), int(q.x_zp), float(q.w_scale),
                                         int(q.w_zp), int(pad_code), gy.ctypes.data, p(out["gx"]), p(out["gx_abs"]),
                                         p(out["gw"]), p(out["gw_abs"]))
    if rc:
        raise RuntimeError("ax_oracle_conv2d_backward failed: %d" % rc)
    return out


def threads() -> int:
    return int(lib().ax_oracle_threads())
