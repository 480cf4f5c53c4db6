"""ctypes binding of libaxconv.so: the same entry points as include/axconv.h.

Only argument marshalling happens here.  Tensors are torch CUDA tensors (torch provides
device memory and the stream); every step of the layer runs in the HIP kernels.  There is
no fallback: a missing library raises at first use.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaxconv.so")

_lib = None


class AxError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("axconv error %d: %s" % (code, text))
        self.code = code


class ax_quant_t(ctypes.Structure):
    _fields_ = [
        ("x_scale", ctypes.c_float),
        ("x_zp", ctypes.c_int32),
        ("w_scale", ctypes.c_float),
        ("w_zp", ctypes.c_int32),
        ("pad_code", ctypes.c_int32),
    ]


EXPORTS = [
    "ax_conv2d", "ax_conv2d_workspace_bytes", "ax_dense", "ax_dense_workspace_bytes", "ax_strerror",
    "ax_version", "ax_set_option", "ax_get_option", "ax_probe_lds_gather", "ax_probe_copy", "ax_probe_mac", "ax_last_kernel_ms", "ax_conv2d_plan",
    "ax_range_f32", "ax_range_workspace_bytes", "ax_quantize_f32", "ax_conv2d_f32", "ax_conv2d_f32_workspace_bytes",
    "ax_dense_f32", "ax_dense_f32_workspace_bytes", "ax_conv2d_ex", "ax_conv2d_ex_workspace_bytes",
    "ax_conv2d_multi_lut", "ax_conv2d_multi_lut_workspace_bytes", "ax_conv2d_f32_ex", "ax_conv2d_f32_ex_workspace_bytes",
]


AX_PAD_DEFAULT = -(1 << 31)


class ax_conv_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "H", "W", "Cin", "KH", "KW", "Cout", "stride_h", "stride_w", "pad_h", "pad_w", "dilation_h", "dilation_w",
        "depthwise", "signed_codes")]


def lib():
    """Load libaxconv.so (built beforehand by paper_2002_09481_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libaxconv.so is not built: run `python -m paper_2002_09481_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.ax_conv2d.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci,
                            ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d.restype = ci
    L.ax_conv2d_workspace_bytes.argtypes = [ci] * 11
    L.ax_conv2d_workspace_bytes.restype = sz
    L.ax_dense.argtypes = [vp, ci, ci, vp, ci, vp, ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_dense.restype = ci
    L.ax_dense_workspace_bytes.argtypes = [ci, ci, ci]
    L.ax_dense_workspace_bytes.restype = sz
    L.ax_strerror.argtypes = [ci]
    L.ax_strerror.restype = ctypes.c_char_p
    L.ax_version.argtypes = []
    L.ax_version.restype = ci
    L.ax_set_option.argtypes = [ctypes.c_char_p, ci]
    L.ax_set_option.restype = ci
    L.ax_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(ci)]
    L.ax_get_option.restype = ci
    dp = ctypes.POINTER(ctypes.c_double)
    L.ax_probe_lds_gather.argtypes = [ci, ci, ci, ci, ci, dp, dp, dp, ctypes.POINTER(ci), vp]
    L.ax_probe_lds_gather.restype = ci
    L.ax_probe_mac.argtypes = [ci, ci, ci, ci, dp, dp, vp]
    L.ax_probe_mac.restype = ci
    ip = ctypes.POINTER(ci)
    L.ax_conv2d_plan.argtypes = [ci] * 11 + [ip, ip, ip, ip]
    L.ax_conv2d_plan.restype = ci
    L.ax_last_kernel_ms.argtypes = [ctypes.POINTER(ctypes.c_float)]
    L.ax_last_kernel_ms.restype = ci
    L.ax_probe_copy.argtypes = [vp, vp, sz, vp]
    L.ax_probe_copy.restype = ci
    L.ax_conv2d_multi_lut.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci,
                                      ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d_multi_lut.restype = ci
    L.ax_conv2d_multi_lut_workspace_bytes.argtypes = [ci] * 12
    L.ax_conv2d_multi_lut_workspace_bytes.restype = sz
    L.ax_conv2d_f32_ex.argtypes = [ctypes.POINTER(ax_conv_desc_t), vp, vp, vp, vp, vp, ci, ci, vp, vp, vp, sz, vp]
    L.ax_conv2d_f32_ex.restype = ci
    L.ax_conv2d_f32_ex_workspace_bytes.argtypes = [ctypes.POINTER(ax_conv_desc_t)]
    L.ax_conv2d_f32_ex_workspace_bytes.restype = sz
    L.ax_conv2d_ex.argtypes = [ctypes.POINTER(ax_conv_desc_t), vp, vp, vp, ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d_ex.restype = ci
    L.ax_conv2d_ex_workspace_bytes.argtypes = [ctypes.POINTER(ax_conv_desc_t)]
    L.ax_conv2d_ex_workspace_bytes.restype = sz
    L.ax_range_f32.argtypes = [vp, sz, ci, vp, vp, sz, vp]
    L.ax_range_f32.restype = ci
    L.ax_range_workspace_bytes.argtypes = [sz]
    L.ax_range_workspace_bytes.restype = sz
    L.ax_quantize_f32.argtypes = [vp, sz, vp, ci, ci, vp, vp, vp]
    L.ax_quantize_f32.restype = ci
    L.ax_conv2d_f32.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, vp, vp, ci, ci, vp, vp, vp,
                                sz, vp]
    L.ax_conv2d_f32.restype = ci
    L.ax_conv2d_f32_workspace_bytes.argtypes = [ci] * 11
    L.ax_conv2d_f32_workspace_bytes.restype = sz
    L.ax_dense_f32.argtypes = [vp, ci, ci, vp, ci, vp, vp, vp, ci, ci, vp, vp, vp, sz, vp]
    L.ax_dense_f32.restype = ci
    L.ax_dense_f32_workspace_bytes.argtypes = [ci, ci, ci]
    L.ax_dense_f32_workspace_bytes.restype = sz
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        raise AxError(rc, lib().ax_strerror(rc).decode())


def ax_strerror(code: int) -> str:
    return lib().ax_strerror(code).decode()


def ax_version() -> int:
    return int(lib().ax_version())


def ax_set_option(name: str, value: int) -> None:
    _check(lib().ax_set_option(name.encode(), int(value)))


def ax_get_option(name: str) -> int:
    v = ctypes.c_int(0)
    _check(lib().ax_get_option(name.encode(), ctypes.byref(v)))
    return v.value


def ax_conv2d_plan(x_shape, w_shape, stride=1, pad=0) -> dict:
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, Cout = [int(v) for v in w_shape]
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    out = [ctypes.c_int(0) for _ in range(4)]
    _check(lib().ax_conv2d_plan(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, *[ctypes.byref(o) for o in out]))
    return {"variant": out[0].value, "tile": out[1].value, "workgroups": out[2].value, "pieces": out[3].value}


def ax_last_kernel_ms() -> float:
    v = ctypes.c_float(0.0)
    _check(lib().ax_last_kernel_ms(ctypes.byref(v)))
    return float(v.value)


def _quant(q) -> ax_quant_t:
    return ax_quant_t(float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), int(q.pad_code))


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t


def _pair(v) -> Tuple[int, int]:
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def ax_conv2d_workspace_bytes(x_shape, w_shape, stride=1, pad=0) -> int:
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, Cout = [int(v) for v in w_shape]
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    return int(lib().ax_conv2d_workspace_bytes(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw))


def ax_dense_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().ax_dense_workspace_bytes(int(M), int(K), int(N)))


def ax_conv2d(x, w, lut, stride, pad, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """Enqueue one layer.  x: uint8 [N,H,W,Cin]; w: uint8 [KH,KW,Cin,Cout]; lut: int16/uint16
    [65536] (bit pattern of the uint16 entries); acc_out: int32 [N,OH,OW,Cout]; y_out: float32.
    Missing outputs / workspace are allocated with torch (the C call itself never allocates).
    Returns (acc_out, y_out)."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    if lut.dtype not in (torch.int16, torch.uint16):
        raise TypeError("lut must be a 16-bit integer tensor")
    _dev(lut, lut.dtype, "lut")
    if lut.numel() != 65536:
        raise ValueError("lut must have 65536 entries")
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    OH = (H + 2 * ph - KH) // sh + 1
    OW = (W + 2 * pw - KW) // sw + 1
    if OH <= 0 or OW <= 0:
        _check(-2)
    if acc_out is None:
        acc_out = torch.empty((N, OH, OW, Cout), dtype=torch.int32, device=x.device)
    if y_out is None:
        y_out = torch.empty((N, OH, OW, Cout), dtype=torch.float32, device=x.device)
    if acc_out is not False:
        _dev(acc_out, torch.int32, "acc_out")
    if y_out is not False:
        _dev(y_out, torch.float32, "y_out")
    for o in (acc_out, y_out):
        if o is not False and o.numel() != N * OH * OW * Cout:
            raise ValueError("output tensor has the wrong number of elements")
    if workspace is None:  # (a workspace handed in is checked by the C call itself)
        need = int(L.ax_conv2d_workspace_bytes(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw))
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    rc = L.ax_conv2d(_ptr(x), N, H, W, Cin, _ptr(w), KH, KW, Cout, _ptr(lut), sh, sw, ph, pw, ctypes.byref(qs),
                     _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                     _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_dense(x, w, lut, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """x: uint8 [M,K]; w: uint8 [K,N]; outputs [M,N]."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    if lut.dtype not in (torch.int16, torch.uint16):
        raise TypeError("lut must be a 16-bit integer tensor")
    _dev(lut, lut.dtype, "lut")
    if lut.numel() != 65536:
        raise ValueError("lut must have 65536 entries")
    if x.dim() != 2 or w.dim() != 2 or w.shape[0] != x.shape[1]:
        raise ValueError("x must be [M,K] and w [K,N]")
    M, K = x.shape
    N = w.shape[1]
    if acc_out is None:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=x.device)
    if y_out is None:
        y_out = torch.empty((M, N), dtype=torch.float32, device=x.device)
    if acc_out is not False:
        _dev(acc_out, torch.int32, "acc_out")
    if y_out is not False:
        _dev(y_out, torch.float32, "y_out")
    if workspace is None:
        need = int(L.ax_dense_workspace_bytes(M, K, N))
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    rc = L.ax_dense(_ptr(x), M, K, _ptr(w), N, _ptr(lut), ctypes.byref(qs),
                    _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                    _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_multi_lut_workspace_bytes(x_shape, w_shape, num_luts, stride=1, pad=0) -> int:
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, Cout = [int(v) for v in w_shape]
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    return int(lib().ax_conv2d_multi_lut_workspace_bytes(N, H, W, Cin, KH, KW, Cout, int(num_luts), sh, sw, ph, pw))


def ax_conv2d_multi_lut(x, w, luts, stride, pad, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """One layer against T tables.  luts: 16-bit integer CUDA tensor [T, 65536]; outputs
    [T, N, OH, OW, Cout].  Returns (acc_out, y_out); pass False to skip one of them."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    if luts.dtype not in (torch.int16, torch.uint16):
        raise TypeError("luts must be a 16-bit integer tensor")
    _dev(luts, luts.dtype, "luts")
    if luts.dim() != 2 or luts.shape[1] != 65536:
        raise ValueError("luts must be [T, 65536]")
    T = int(luts.shape[0])
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    OH = (H + 2 * ph - KH) // sh + 1
    OW = (W + 2 * pw - KW) // sw + 1
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((T, N, OH, OW, Cout), x.device, acc_out, y_out)
    if workspace is None:
        need = int(L.ax_conv2d_multi_lut_workspace_bytes(N, H, W, Cin, KH, KW, Cout, T, sh, sw, ph, pw))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    rc = L.ax_conv2d_multi_lut(_ptr(x), N, H, W, Cin, _ptr(w), KH, KW, Cout, _ptr(luts), T, sh, sw, ph, pw,
                               ctypes.byref(qs), _ptr(None if acc_out is False else acc_out),
                               _ptr(None if y_out is False else y_out), _ptr(workspace), workspace.numel(),
                               ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_ex(x, w, lut, stride, pad, q, dilation=1, depthwise=False, acc_out=None, y_out=None, workspace=None,
                 stream=None):
    """Operator variants.  Signed form: x, w int8 and lut int16 (chosen by x.dtype).  Depthwise:
    w is [KH,KW,Cin,mult].  q.pad_code None selects the zero point.  Returns (acc_out, y_out)."""
    L = lib()
    signed = x.dtype == torch.int8
    cdt = torch.int8 if signed else torch.uint8
    _dev(x, cdt, "x")
    _dev(w, cdt, "w")
    if lut.dtype not in (torch.int16, torch.uint16):
        raise TypeError("lut must be a 16-bit integer tensor")
    _dev(lut, lut.dtype, "lut")
    if lut.numel() != 65536:
        raise ValueError("lut must have 65536 entries")
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout] (or [KH,KW,Cin,mult])")
    N, H, W, Cin = x.shape
    KH, KW, _, last = w.shape
    Cout = Cin * last if depthwise else last
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dilation)
    desc = ax_conv_desc_t(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, int(bool(depthwise)), int(signed))
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((N, OH, OW, Cout), x.device, acc_out, y_out)
    if workspace is None:
        need = int(L.ax_conv2d_ex_workspace_bytes(ctypes.byref(desc)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    pad_code = AX_PAD_DEFAULT if q.pad_code is None else int(q.pad_code)
    qs = ax_quant_t(float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), pad_code)
    rc = L.ax_conv2d_ex(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(lut), ctypes.byref(qs),
                        _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                        _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_range_workspace_bytes(n: int) -> int:
    return int(lib().ax_range_workspace_bytes(int(n)))


def ax_range_f32(x, relu=False, range_out=None, workspace=None, stream=None):
    """(min, max) of a float32 CUDA tensor into a float32 CUDA tensor of two."""
    L = lib()
    _dev(x, torch.float32, "x")
    if range_out is None:
        range_out = torch.empty(2, dtype=torch.float32, device=x.device)
    _dev(range_out, torch.float32, "range_out")
    if workspace is None:
        workspace = torch.empty(int(L.ax_range_workspace_bytes(x.numel())), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    _check(L.ax_range_f32(_ptr(x), x.numel(), int(bool(relu)), _ptr(range_out), _ptr(workspace), workspace.numel(),
                          ctypes.c_void_p(_stream_ptr(stream))))
    return range_out


def ax_quantize_f32(x, rng, relu=False, round_mode=0, codes_out=None, coeffs_out=None, stream=None):
    """Codes of a float32 CUDA tensor for the range `rng` (float32 CUDA tensor of two).
    coeffs_out: int32 CUDA tensor of two receiving the bit pattern of alpha and the value of
    beta (allocated when None).  Returns (codes_out, coeffs_out)."""
    L = lib()
    _dev(x, torch.float32, "x")
    _dev(rng, torch.float32, "range")
    if rng.numel() != 2:
        raise ValueError("range must hold two floats")
    if codes_out is None:
        codes_out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _dev(codes_out, torch.uint8, "codes_out")
    if codes_out.numel() != x.numel():
        raise ValueError("codes_out has the wrong number of elements")
    if coeffs_out is None:
        coeffs_out = torch.empty(2, dtype=torch.int32, device=x.device)
    _dev(coeffs_out, torch.int32, "coeffs_out")
    _check(L.ax_quantize_f32(_ptr(x), x.numel(), _ptr(rng), int(bool(relu)), int(round_mode), _ptr(codes_out),
                             _ptr(coeffs_out), ctypes.c_void_p(_stream_ptr(stream))))
    return codes_out, coeffs_out


def ax_conv2d_f32_workspace_bytes(x_shape, w_shape, stride=1, pad=0) -> int:
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, Cout = [int(v) for v in w_shape]
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    return int(lib().ax_conv2d_f32_workspace_bytes(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw))


def ax_dense_f32_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(lib().ax_dense_f32_workspace_bytes(int(M), int(K), int(N)))


def _f32_common(x, w, lut, x_range, w_range):
    _dev(x, torch.float32, "x")
    _dev(w, torch.float32, "w")
    for r, name in ((x_range, "x_range"), (w_range, "w_range")):
        if r is None:  # the layer takes the range itself
            continue
        _dev(r, torch.float32, name)
        if r.numel() != 2:
            raise ValueError("ranges must hold two floats")
    if lut.dtype not in (torch.int16, torch.uint16):
        raise TypeError("lut must be a 16-bit integer tensor")
    _dev(lut, lut.dtype, "lut")
    if lut.numel() != 65536:
        raise ValueError("lut must have 65536 entries")


def _outs(shape, device, acc_out, y_out):
    if acc_out is None:
        acc_out = torch.empty(shape, dtype=torch.int32, device=device)
    if y_out is None:
        y_out = torch.empty(shape, dtype=torch.float32, device=device)
    n = 1
    for v in shape:
        n *= int(v)
    if acc_out is not False:
        _dev(acc_out, torch.int32, "acc_out")
    if y_out is not False:
        _dev(y_out, torch.float32, "y_out")
    for o in (acc_out, y_out):
        if o is not False and o.numel() != n:
            raise ValueError("output tensor has the wrong number of elements")
    return acc_out, y_out


def ax_conv2d_f32(x, w, lut, stride, pad, x_range=None, w_range=None, relu=False, round_mode=0, acc_out=None, y_out=None,
                  workspace=None, stream=None):
    """Float layer.  x: float32 [N,H,W,Cin]; w: float32 [KH,KW,Cin,Cout]; ranges: float32 CUDA
    tensors of two, or None to let the layer take the range of that tensor.  Returns (acc_out, y_out); pass False to skip one of them."""
    L = lib()
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    OH = (H + 2 * ph - KH) // sh + 1
    OW = (W + 2 * pw - KW) // sw + 1
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((N, OH, OW, Cout), x.device, acc_out, y_out)
    if workspace is None:
        need = int(L.ax_conv2d_f32_workspace_bytes(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw))
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_conv2d_f32(_ptr(x), N, H, W, Cin, _ptr(w), KH, KW, Cout, _ptr(lut), sh, sw, ph, pw, _ptr(x_range),
                         _ptr(w_range), int(bool(relu)), int(round_mode),
                         _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                         _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_f32_ex(x, w, lut, stride, pad, x_range=None, w_range=None, relu=False, round_mode=0, dilation=1,
                     depthwise=False, signed=False, acc_out=None, y_out=None, workspace=None, stream=None):
    """Float layer with dilation / signed codes / depthwise filters (w [KH,KW,Cin,mult]).
    Returns (acc_out, y_out); pass False to skip one of them."""
    L = lib()
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout] (or [KH,KW,Cin,mult])")
    N, H, W, Cin = x.shape
    KH, KW, _, last = w.shape
    Cout = Cin * last if depthwise else last
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dilation)
    desc = ax_conv_desc_t(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, int(bool(depthwise)), int(bool(signed)))
    OH = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((N, OH, OW, Cout), x.device, acc_out, y_out)
    if workspace is None:
        need = int(L.ax_conv2d_f32_ex_workspace_bytes(ctypes.byref(desc)))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_conv2d_f32_ex(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(lut), _ptr(x_range), _ptr(w_range),
                            int(bool(relu)), int(round_mode), _ptr(None if acc_out is False else acc_out),
                            _ptr(None if y_out is False else y_out), _ptr(workspace), workspace.numel(),
                            ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_dense_f32(x, w, lut, x_range=None, w_range=None, relu=False, round_mode=0, acc_out=None, y_out=None, workspace=None,
                 stream=None):
    """x: float32 [M,K]; w: float32 [K,N]; outputs [M,N]."""
    L = lib()
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 2 or w.dim() != 2 or w.shape[0] != x.shape[1]:
        raise ValueError("x must be [M,K] and w [K,N]")
    M, K = x.shape
    N = w.shape[1]
    acc_out, y_out = _outs((M, N), x.device, acc_out, y_out)
    if workspace is None:
        workspace = torch.empty(int(L.ax_dense_f32_workspace_bytes(M, K, N)), dtype=torch.uint8, device=x.device)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_dense_f32(_ptr(x), M, K, _ptr(w), N, _ptr(lut), _ptr(x_range), _ptr(w_range), int(bool(relu)),
                        int(round_mode), _ptr(None if acc_out is False else acc_out),
                        _ptr(None if y_out is False else y_out), _ptr(workspace), workspace.numel(),
                        ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_probe_lds_gather(width_bytes: int, pattern: int, table_bytes: int, threads: int = 1024, iters: int = 2000,
                        stream=None) -> dict:
    wr, cy, sec = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    wgs = ctypes.c_int()
    rc = lib().ax_probe_lds_gather(width_bytes, pattern, table_bytes, threads, iters, ctypes.byref(wr),
                                   ctypes.byref(cy), ctypes.byref(sec), ctypes.byref(wgs),
                                   ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return {"wave_reads": wr.value, "cycles": cy.value, "seconds": sec.value, "workgroups": wgs.value}


def ax_probe_mac(mode: int, pattern: int = 1, iters: int = 200, wgs_per_cu: int = 1, stream=None) -> dict:
    ops, sec = ctypes.c_double(), ctypes.c_double()
    _check(lib().ax_probe_mac(mode, pattern, iters, wgs_per_cu, ctypes.byref(ops), ctypes.byref(sec),
                              ctypes.c_void_p(_stream_ptr(stream))))
    return {"ops": ops.value, "seconds": sec.value, "ops_per_s": ops.value / sec.value}


def ax_probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().ax_probe_copy(_ptr(dst), _ptr(src), nbytes, ctypes.c_void_p(_stream_ptr(stream))))


def lut_to_device(lut_np, device="cuda") -> torch.Tensor:
    """uint16 (or, for signed multipliers, int16) numpy table -> device tensor holding the same
    bit patterns."""
    import numpy as np

    a = np.ascontiguousarray(lut_np)
    if a.dtype != np.int16:
        a = np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(a.reshape(-1).copy()).to(device)
