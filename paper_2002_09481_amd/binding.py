"""ctypes binding of libaxconv.so: the same entry points as include/axconv.h and
include/axconv_probe.h.

Only argument marshalling happens here.  Tensors are torch CUDA tensors (torch provides
device memory and the stream); every step of the layer runs in the HIP kernels.  There is
no fallback: a missing library raises at first use.

The library itself keeps no options: tuning overrides travel with each call as an ax_tune_t.
ax_set_option / ax_get_option below only keep this module's default for that argument (the
tests use them to force every kernel path); calls made while a default is set go through the
entry points that accept a tune (ax_conv2d_ex, ax_conv2d_f32_ex, the layer handles).
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


EXPORTS = [  # include/axconv.h
    "ax_conv2d", "ax_conv2d_workspace_bytes", "ax_dense", "ax_dense_workspace_bytes", "ax_strerror",
    "ax_conv2d_transpose", "ax_conv2d_transpose_workspace_bytes", "ax_version", "ax_range_f32", "ax_range_workspace_bytes", "ax_quantize_f32", "ax_conv2d_f32",
    "ax_conv2d_f32_workspace_bytes", "ax_dense_f32", "ax_dense_f32_workspace_bytes", "ax_conv2d_ex",
    "ax_conv2d_ex_workspace_bytes", "ax_conv2d_multi_lut", "ax_conv2d_multi_lut_workspace_bytes", "ax_conv2d_f32_ex",
    "ax_conv2d_f32_ex_workspace_bytes", "ax_layer_create", "ax_layer_destroy", "ax_layer_prepared_bytes",
    "ax_layer_workspace_bytes", "ax_layer_prepare", "ax_layer_run", "ax_layer_plan", "ax_layer_plan_paths", "ax_layer_run_static",
    "ax_static_scratch_bytes", "ax_conv2d_backward", "ax_conv2d_backward_workspace_bytes",
]
PROBE_EXPORTS = [  # include/axconv_probe.h
    "ax_probe_lds_gather", "ax_probe_copy", "ax_probe_mac", "ax_probe_layer_kernel_ms",
]


AX_PAD_DEFAULT = -(1 << 31)


class ax_tune_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("variant", "split_k", "tile", "row_tiles", "share_order", "combine", "tables")]


class ax_conv_desc_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "H", "W", "Cin", "KH", "KW", "Cout", "stride_h", "stride_w", "pad_h", "pad_w", "dilation_h", "dilation_w",
        "depthwise", "signed_codes", "groups")]


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
    dp = ctypes.POINTER(ctypes.c_double)
    L.ax_probe_lds_gather.argtypes = [ci, ci, ci, ci, ci, dp, dp, dp, ctypes.POINTER(ci), vp]
    L.ax_probe_lds_gather.restype = ci
    L.ax_probe_mac.argtypes = [ci, ci, ci, ci, dp, dp, vp]
    L.ax_probe_mac.restype = ci
    ip = ctypes.POINTER(ci)
    tp = ctypes.POINTER(ax_tune_t)
    descp = ctypes.POINTER(ax_conv_desc_t)
    L.ax_layer_create.argtypes = [descp, ci, ctypes.POINTER(ax_quant_t), tp, ctypes.POINTER(vp)]
    L.ax_layer_create.restype = ci
    L.ax_layer_destroy.argtypes = [vp]
    L.ax_layer_destroy.restype = None
    L.ax_layer_prepared_bytes.argtypes = [vp]
    L.ax_layer_prepared_bytes.restype = sz
    L.ax_layer_workspace_bytes.argtypes = [vp]
    L.ax_layer_workspace_bytes.restype = sz
    L.ax_layer_prepare.argtypes = [vp, vp, vp, vp, sz, vp]
    L.ax_layer_prepare.restype = ci
    L.ax_layer_run.argtypes = [vp, vp, vp, vp, vp, sz, vp]
    L.ax_layer_run.restype = ci
    L.ax_layer_plan.argtypes = [vp, ip, ip, ip, ip]
    L.ax_layer_plan.restype = ci
    L.ax_layer_plan_paths.argtypes = [vp, ip, ip]
    L.ax_layer_plan_paths.restype = ci
    L.ax_layer_run_static.argtypes = [vp, vp, vp, vp, vp]
    L.ax_layer_run_static.restype = ci
    L.ax_static_scratch_bytes.argtypes = []
    L.ax_static_scratch_bytes.restype = sz
    L.ax_conv2d_backward.argtypes = [descp, ctypes.POINTER(ax_quant_t), vp, vp, vp, vp, vp, vp, sz, vp]
    L.ax_conv2d_backward.restype = ci
    L.ax_conv2d_backward_workspace_bytes.argtypes = [descp]
    L.ax_conv2d_backward_workspace_bytes.restype = sz
    L.ax_probe_layer_kernel_ms.argtypes = [vp, vp, vp, vp, vp, sz, ci, ctypes.POINTER(ctypes.c_float), vp]
    L.ax_probe_layer_kernel_ms.restype = ci
    L.ax_probe_copy.argtypes = [vp, vp, sz, vp]
    L.ax_probe_copy.restype = ci
    L.ax_conv2d_multi_lut.argtypes = [vp, ci, ci, ci, ci, vp, ci, ci, ci, vp, ci, ci, ci, ci, ci,
                                      ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d_multi_lut.restype = ci
    L.ax_conv2d_multi_lut_workspace_bytes.argtypes = [ci] * 12
    L.ax_conv2d_multi_lut_workspace_bytes.restype = sz
    L.ax_conv2d_f32_ex.argtypes = [descp, tp, vp, vp, vp, vp, vp, ci, ci, vp, vp, vp, sz, vp]
    L.ax_conv2d_f32_ex.restype = ci
    L.ax_conv2d_f32_ex_workspace_bytes.argtypes = [descp, tp]
    L.ax_conv2d_f32_ex_workspace_bytes.restype = sz
    L.ax_conv2d_ex.argtypes = [descp, tp, vp, vp, vp, ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d_ex.restype = ci
    L.ax_conv2d_ex_workspace_bytes.argtypes = [descp, tp]
    L.ax_conv2d_ex_workspace_bytes.restype = sz
    L.ax_conv2d_transpose.argtypes = [descp, tp, vp, vp, vp, ctypes.POINTER(ax_quant_t), vp, vp, vp, sz, vp]
    L.ax_conv2d_transpose_workspace_bytes.argtypes = [descp, tp]
    L.ax_conv2d_transpose_workspace_bytes.restype = sz
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


def ax_static_scratch_bytes() -> int:
    return int(lib().ax_static_scratch_bytes())


def ax_strerror(code: int) -> str:
    return lib().ax_strerror(code).decode()


def ax_version() -> int:
    return int(lib().ax_version())


_TUNE_FIELDS = ("variant", "split_k", "tile", "row_tiles", "share_order", "combine", "tables")
_tune = {n: 0 for n in _TUNE_FIELDS}  # this module's default ax_tune_t (all zero = automatic)


def _tune_arg(tune=None):
    """ctypes argument for a `const ax_tune_t*` parameter: NULL when everything is automatic."""
    t = _tune if tune is None else tune
    if not any(t.get(n, 0) for n in _TUNE_FIELDS):
        return None
    return ctypes.byref(ax_tune_t(*[int(t.get(n, 0)) for n in _TUNE_FIELDS]))


def ax_set_option(name: str, value: int) -> None:
    """Set one field of the module's default tune; the library checks the value's range."""
    if name not in _tune:
        raise AxError(-8, lib().ax_strerror(-8).decode())
    trial = dict(_tune)
    trial[name] = int(value)
    if not -(1 << 31) <= trial[name] < (1 << 31):
        raise AxError(-8, lib().ax_strerror(-8).decode())
    desc = ax_conv_desc_t(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1, 0, 0)
    q = ax_quant_t(1.0, 0, 1.0, 0, -1)
    h = ctypes.c_void_p()
    _check(lib().ax_layer_create(ctypes.byref(desc), 1, ctypes.byref(q), _tune_arg(trial), ctypes.byref(h)))
    lib().ax_layer_destroy(h)
    _tune[name] = trial[name]


def ax_get_option(name: str) -> int:
    if name not in _tune:
        raise AxError(-8, lib().ax_strerror(-8).decode())
    return _tune[name]


def ax_conv2d_plan(x_shape, w_shape, stride=1, pad=0, num_luts=1) -> dict:
    """What a layer of this geometry runs under the module's default tune (host arithmetic)."""
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, Cout = [int(v) for v in w_shape]
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    desc = ax_conv_desc_t(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, 1, 1, 0, 0)
    with AxLayer(desc, ax_quant_t(1.0, 0, 1.0, 0, -1), num_luts) as layer:
        return layer.plan()


def _quant(q) -> ax_quant_t:
    pad_code = AX_PAD_DEFAULT if q.pad_code is None else int(q.pad_code)
    return ax_quant_t(float(q.x_scale), int(q.x_zp), float(q.w_scale), int(q.w_zp), pad_code)


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


def _workspace(need: int, device, stream) -> torch.Tensor:
    """Temporary scratch for one call.  torch's allocator hands memory back to the current
    stream's pool when the tensor dies: for a call on another stream the allocation is tied to
    that stream as well, so that it is not reused while the kernels still run."""
    ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device=device)
    if stream is not None:
        ws.record_stream(stream)
    return ws


def _conv_desc(x_shape, w_shape, stride, pad, dilation=1, depthwise=False, signed=False, groups=1) -> ax_conv_desc_t:
    N, H, W, Cin = [int(v) for v in x_shape]
    KH, KW, _, last = [int(v) for v in w_shape]
    Cout = Cin * last if depthwise else last
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dilation)
    return ax_conv_desc_t(N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, int(bool(depthwise)), int(bool(signed)),
                          int(groups))


def _dense_desc(M: int, K: int, N: int) -> ax_conv_desc_t:
    return ax_conv_desc_t(int(M), 1, 1, int(K), 1, 1, int(N), 1, 1, 0, 0, 1, 1, 0, 0)


def _out_hw(d: ax_conv_desc_t) -> Tuple[int, int]:
    OH = (d.H + 2 * d.pad_h - d.dilation_h * (d.KH - 1) - 1) // d.stride_h + 1
    OW = (d.W + 2 * d.pad_w - d.dilation_w * (d.KW - 1) - 1) // d.stride_w + 1
    return OH, OW


def ax_conv2d_workspace_bytes(x_shape, w_shape, stride=1, pad=0) -> int:
    d = _conv_desc(x_shape, w_shape, stride, pad)
    t = _tune_arg()
    if t is not None:
        return int(lib().ax_conv2d_ex_workspace_bytes(ctypes.byref(d), t))
    return int(lib().ax_conv2d_workspace_bytes(d.N, d.H, d.W, d.Cin, d.KH, d.KW, d.Cout, d.stride_h, d.stride_w,
                                               d.pad_h, d.pad_w))


def ax_dense_workspace_bytes(M: int, K: int, N: int) -> int:
    t = _tune_arg()
    if t is not None:
        return int(lib().ax_conv2d_ex_workspace_bytes(ctypes.byref(_dense_desc(M, K, N)), t))
    return int(lib().ax_dense_workspace_bytes(int(M), int(K), int(N)))


def _check_lut(lut, n_entries=65536):
    if lut.dtype not in (torch.int16, torch.uint16):
        raise TypeError("lut must be a 16-bit integer tensor")
    _dev(lut, lut.dtype, "lut")
    if lut.numel() != n_entries:
        raise ValueError("lut must have %d entries" % n_entries)


def ax_conv2d(x, w, lut, stride, pad, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """Enqueue one layer.  x: uint8 [N,H,W,Cin]; w: uint8 [KH,KW,Cin,Cout]; lut: int16/uint16
    [65536] (bit pattern of the uint16 entries); acc_out: int32 [N,OH,OW,Cout]; y_out: float32.
    Missing outputs / workspace are allocated with torch (the C call itself never allocates).
    Returns (acc_out, y_out)."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    _check_lut(lut)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    d = _conv_desc(x.shape, w.shape, stride, pad)
    OH, OW = _out_hw(d)
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((d.N, OH, OW, d.Cout), x.device, acc_out, y_out)
    if workspace is None:  # (a workspace handed in is checked by the C call itself)
        workspace = _workspace(ax_conv2d_workspace_bytes(x.shape, w.shape, stride, pad), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    t = _tune_arg()
    tail = (ctypes.byref(qs), _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
            _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    if t is None:
        rc = L.ax_conv2d(_ptr(x), d.N, d.H, d.W, d.Cin, _ptr(w), d.KH, d.KW, d.Cout, _ptr(lut), d.stride_h, d.stride_w,
                         d.pad_h, d.pad_w, *tail)
    else:
        rc = L.ax_conv2d_ex(ctypes.byref(d), t, _ptr(x), _ptr(w), _ptr(lut), *tail)
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_dense(x, w, lut, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """x: uint8 [M,K]; w: uint8 [K,N]; outputs [M,N]."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    _check_lut(lut)
    if x.dim() != 2 or w.dim() != 2 or w.shape[0] != x.shape[1]:
        raise ValueError("x must be [M,K] and w [K,N]")
    M, K = x.shape
    N = w.shape[1]
    acc_out, y_out = _outs((M, N), x.device, acc_out, y_out)
    if workspace is None:
        workspace = _workspace(ax_dense_workspace_bytes(M, K, N), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    t = _tune_arg()
    tail = (ctypes.byref(qs), _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
            _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    if t is None:
        rc = L.ax_dense(_ptr(x), M, K, _ptr(w), N, _ptr(lut), *tail)
    else:
        rc = L.ax_conv2d_ex(ctypes.byref(_dense_desc(M, K, N)), t, _ptr(x), _ptr(w), _ptr(lut), *tail)
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_multi_lut_workspace_bytes(x_shape, w_shape, num_luts, stride=1, pad=0) -> int:
    d = _conv_desc(x_shape, w_shape, stride, pad)
    return int(lib().ax_conv2d_multi_lut_workspace_bytes(d.N, d.H, d.W, d.Cin, d.KH, d.KW, d.Cout, int(num_luts),
                                                         d.stride_h, d.stride_w, d.pad_h, d.pad_w))


def ax_conv2d_multi_lut(x, w, luts, stride, pad, q, acc_out=None, y_out=None, workspace=None, stream=None):
    """One layer against T tables.  luts: 16-bit integer CUDA tensor [T, 65536]; outputs
    [T, N, OH, OW, Cout].  Returns (acc_out, y_out); pass False to skip one of them.  With a
    default tune set the call goes through a layer handle (the one-call entry takes no tune)."""
    L = lib()
    _dev(x, torch.uint8, "x")
    _dev(w, torch.uint8, "w")
    if luts.dim() != 2 or luts.shape[1] != 65536:
        raise ValueError("luts must be [T, 65536]")
    T = int(luts.shape[0])
    _check_lut(luts, T * 65536)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    d = _conv_desc(x.shape, w.shape, stride, pad)
    OH, OW = _out_hw(d)
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((T, d.N, OH, OW, d.Cout), x.device, acc_out, y_out)
    qs = _quant(q)
    if _tune_arg() is not None:
        with AxLayer(d, qs, T) as layer:
            layer.prepare(w, luts, stream=stream)
            layer.run(x, acc_out, y_out, workspace=workspace, stream=stream)
        return (None if acc_out is False else acc_out), (None if y_out is False else y_out)
    if workspace is None:
        workspace = _workspace(ax_conv2d_multi_lut_workspace_bytes(x.shape, w.shape, T, stride, pad), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_conv2d_multi_lut(_ptr(x), d.N, d.H, d.W, d.Cin, _ptr(w), d.KH, d.KW, d.Cout, _ptr(luts), T, d.stride_h,
                               d.stride_w, d.pad_h, d.pad_w, ctypes.byref(qs),
                               _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                               _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_ex(x, w, lut, stride, pad, q, dilation=1, depthwise=False, acc_out=None, y_out=None, workspace=None,
                 stream=None, groups=1):
    """Operator variants.  Signed form: x, w int8 and lut int16 (chosen by x.dtype).  Depthwise:
    w is [KH,KW,Cin,mult].  Grouped: w is [KH,KW,Cin/groups,Cout].  q.pad_code None selects the
    zero point.  Returns (acc_out, y_out)."""
    L = lib()
    signed = x.dtype == torch.int8
    cdt = torch.int8 if signed else torch.uint8
    _dev(x, cdt, "x")
    _dev(w, cdt, "w")
    _check_lut(lut)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] * int(groups) != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin/groups,Cout] (or [KH,KW,Cin,mult])")
    desc = _conv_desc(x.shape, w.shape, stride, pad, dilation, depthwise, signed, groups)
    OH, OW = _out_hw(desc)
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((desc.N, OH, OW, desc.Cout), x.device, acc_out, y_out)
    t = _tune_arg()
    if workspace is None:
        workspace = _workspace(int(L.ax_conv2d_ex_workspace_bytes(ctypes.byref(desc), t)), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    rc = L.ax_conv2d_ex(ctypes.byref(desc), t, _ptr(x), _ptr(w), _ptr(lut), ctypes.byref(qs),
                        _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                        _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_transpose(x, w, lut, stride, pad, q, dilation=1, acc_out=None, y_out=None, workspace=None, stream=None):
    """Transposed convolution by zero insertion.  x: codes [N,H,W,Cin] (uint8, or int8 for the
    signed form), w: [KH,KW,Cin,Cout].  Returns (acc_out, y_out) of shape [N,OH,OW,Cout] with
    OH = (H-1)*stride + 1 + dilation*(KH-1) - 2*pad."""
    L = lib()
    signed = x.dtype == torch.int8
    cdt = torch.int8 if signed else torch.uint8
    _dev(x, cdt, "x")
    _dev(w, cdt, "w")
    _check_lut(lut)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    desc = _conv_desc(x.shape, w.shape, stride, pad, dilation, False, signed)
    OH = (desc.H - 1) * desc.stride_h + 1 + desc.dilation_h * (desc.KH - 1) - 2 * desc.pad_h
    OW = (desc.W - 1) * desc.stride_w + 1 + desc.dilation_w * (desc.KW - 1) - 2 * desc.pad_w
    if OH <= 0 or OW <= 0:
        _check(-2)
    acc_out, y_out = _outs((desc.N, OH, OW, desc.Cout), x.device, acc_out, y_out)
    t = _tune_arg()
    if workspace is None:
        n = int(L.ax_conv2d_transpose_workspace_bytes(ctypes.byref(desc), t))
        if n == 0:
            _check(-2)
        workspace = _workspace(n, x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    rc = L.ax_conv2d_transpose(ctypes.byref(desc), t, _ptr(x), _ptr(w), _ptr(lut), ctypes.byref(qs),
                               _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                               _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_backward(x, w, gy, stride, pad, q, dilation=1, gx_out=None, gw_out=None, workspace=None, stream=None):
    """Backward pass of a layer (straight-through).  x, w: codes (uint8, or int8 for the signed
    form); gy: float32 [N,OH,OW,Cout].  Returns (gx [N,H,W,Cin], gw [KH,KW,Cin,Cout]) as float32
    tensors; pass False to skip one of them."""
    L = lib()
    signed = x.dtype == torch.int8
    cdt = torch.int8 if signed else torch.uint8
    _dev(x, cdt, "x")
    _dev(w, cdt, "w")
    _dev(gy, torch.float32, "gy")
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    desc = _conv_desc(x.shape, w.shape, stride, pad, dilation, False, signed)
    OH, OW = _out_hw(desc)
    if OH <= 0 or OW <= 0:
        _check(-2)
    if tuple(gy.shape) != (desc.N, OH, OW, desc.Cout):
        raise ValueError("gy must be [N,OH,OW,Cout]")
    if gx_out is None:
        gx_out = torch.empty(x.shape, dtype=torch.float32, device=x.device)
    if gw_out is None:
        gw_out = torch.empty(w.shape, dtype=torch.float32, device=x.device)
    for o, ref, name in ((gx_out, x, "gx_out"), (gw_out, w, "gw_out")):
        if o is not False:
            _dev(o, torch.float32, name)
            if o.numel() != ref.numel():
                raise ValueError("%s has the wrong number of elements" % name)
    if workspace is None:
        workspace = _workspace(int(L.ax_conv2d_backward_workspace_bytes(ctypes.byref(desc))), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    qs = _quant(q)
    _check(L.ax_conv2d_backward(ctypes.byref(desc), ctypes.byref(qs), _ptr(x), _ptr(w), _ptr(gy),
                                _ptr(None if gx_out is False else gx_out), _ptr(None if gw_out is False else gw_out),
                                _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream))))
    return (None if gx_out is False else gx_out), (None if gw_out is False else gw_out)


class AxLayer:
    """A layer handle (ax_layer_*): filters and tables prepared once, then many calls.

    desc: ax_conv_desc_t; q: ax_quant_t or an object with x_scale, x_zp, w_scale, w_zp,
    pad_code (None = zero point); tune: dict with the fields of ax_tune_t (None = the module's
    default).  Device memory (prepared block, workspace) is torch tensors owned by this object
    unless the caller hands tensors in."""

    def __init__(self, desc: ax_conv_desc_t, q, num_luts: int = 1, tune=None):
        self._h = ctypes.c_void_p()
        self.desc = desc
        self.num_luts = int(num_luts)
        qs = q if isinstance(q, ax_quant_t) else _quant(q)
        _check(lib().ax_layer_create(ctypes.byref(desc), self.num_luts, ctypes.byref(qs), _tune_arg(tune),
                                     ctypes.byref(self._h)))
        self._keep = None  # tensors the handle's device pointers refer to
        self._ws = None

    def close(self):
        if self._h and _lib is not None:
            _lib.ax_layer_destroy(self._h)
        self._h = ctypes.c_void_p()
        self._keep = None
        self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the module's globals may be gone
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    @property
    def prepared_bytes(self) -> int:
        return int(lib().ax_layer_prepared_bytes(self._h))

    @property
    def workspace_bytes(self) -> int:
        return int(lib().ax_layer_workspace_bytes(self._h))

    def out_shape(self):
        OH, OW = _out_hw(self.desc)
        shape = (self.desc.N, OH, OW, self.desc.Cout)
        return shape if self.num_luts == 1 else (self.num_luts,) + shape

    def plan(self) -> dict:
        out = [ctypes.c_int(0) for _ in range(4)]
        _check(lib().ax_layer_plan(self._h, *[ctypes.byref(o) for o in out]))
        paths = [ctypes.c_int(0) for _ in range(2)]
        _check(lib().ax_layer_plan_paths(self._h, *[ctypes.byref(o) for o in paths]))
        return {"variant": out[0].value, "tile": out[1].value, "workgroups": out[2].value, "pieces": out[3].value,
                "combine": paths[0].value, "tables": paths[1].value}

    def prepare(self, w, luts, prepared=None, stream=None):
        cdt = torch.int8 if self.desc.signed_codes else torch.uint8
        _dev(w, cdt, "w")
        _check_lut(luts, self.num_luts * 65536)
        if prepared is None:
            prepared = torch.empty(max(self.prepared_bytes, 256), dtype=torch.uint8, device=w.device)
        _dev(prepared, torch.uint8, "prepared")
        _check(lib().ax_layer_prepare(self._h, _ptr(w), _ptr(luts), _ptr(prepared), prepared.numel(),
                                      ctypes.c_void_p(_stream_ptr(stream))))
        self._keep = (w, luts, prepared)
        return prepared

    def _args(self, x, acc_out, y_out, workspace, stream):
        cdt = torch.int8 if self.desc.signed_codes else torch.uint8
        _dev(x, cdt, "x")
        acc_out, y_out = _outs(self.out_shape(), x.device, acc_out, y_out)
        if workspace is None:
            if self._ws is None or self._ws.device != x.device:
                self._ws = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8, device=x.device)
            workspace = self._ws
            if stream is not None:
                workspace.record_stream(stream)
        _dev(workspace, torch.uint8, "workspace")
        return acc_out, y_out, workspace

    def run(self, x, acc_out=None, y_out=None, workspace=None, stream=None):
        acc_out, y_out, workspace = self._args(x, acc_out, y_out, workspace, stream)
        _check(lib().ax_layer_run(self._h, _ptr(x), _ptr(None if acc_out is False else acc_out),
                                  _ptr(None if y_out is False else y_out), _ptr(workspace), workspace.numel(),
                                  ctypes.c_void_p(_stream_ptr(stream))))
        return (None if acc_out is False else acc_out), (None if y_out is False else y_out)

    def run_static(self, x, acc_out, y_out, stream=None):
        """ax_layer_run_static: scratch from the library's static device array; nothing is
        allocated, so the outputs must be handed in (False skips one of them)."""
        cdt = torch.int8 if self.desc.signed_codes else torch.uint8
        _dev(x, cdt, "x")
        if acc_out is None or y_out is None:
            raise ValueError("run_static allocates nothing: pass acc_out and y_out (False to skip one)")
        acc_out, y_out = _outs(self.out_shape(), x.device, acc_out, y_out)
        _check(lib().ax_layer_run_static(self._h, _ptr(x), _ptr(None if acc_out is False else acc_out),
                                         _ptr(None if y_out is False else y_out),
                                         ctypes.c_void_p(_stream_ptr(stream))))
        return (None if acc_out is False else acc_out), (None if y_out is False else y_out)

    def kernel_ms(self, x, acc_out=None, y_out=None, workspace=None, reps: int = 8, stream=None) -> float:
        """ax_probe_layer_kernel_ms: duration of one launch of the layer's main kernel."""
        acc_out, y_out, workspace = self._args(x, acc_out, y_out, workspace, stream)
        ms = ctypes.c_float(0.0)
        _check(lib().ax_probe_layer_kernel_ms(self._h, _ptr(x), _ptr(None if acc_out is False else acc_out),
                                              _ptr(None if y_out is False else y_out), _ptr(workspace),
                                              workspace.numel(), int(reps), ctypes.byref(ms),
                                              ctypes.c_void_p(_stream_ptr(stream))))
        return float(ms.value)


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
    d = _conv_desc(x_shape, w_shape, stride, pad)
    t = _tune_arg()
    if t is not None:
        return int(lib().ax_conv2d_f32_ex_workspace_bytes(ctypes.byref(d), t))
    return int(lib().ax_conv2d_f32_workspace_bytes(d.N, d.H, d.W, d.Cin, d.KH, d.KW, d.Cout, d.stride_h, d.stride_w,
                                                   d.pad_h, d.pad_w))


def ax_dense_f32_workspace_bytes(M: int, K: int, N: int) -> int:
    t = _tune_arg()
    if t is not None:
        return int(lib().ax_conv2d_f32_ex_workspace_bytes(ctypes.byref(_dense_desc(M, K, N)), t))
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
    _check_lut(lut)


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


def _f32_ex(desc, x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace, stream, out_shape):
    L = lib()
    acc_out, y_out = _outs(out_shape, x.device, acc_out, y_out)
    t = _tune_arg()
    if workspace is None:
        workspace = _workspace(int(L.ax_conv2d_f32_ex_workspace_bytes(ctypes.byref(desc), t)), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_conv2d_f32_ex(ctypes.byref(desc), t, _ptr(x), _ptr(w), _ptr(lut), _ptr(x_range), _ptr(w_range),
                            int(bool(relu)), int(round_mode), _ptr(None if acc_out is False else acc_out),
                            _ptr(None if y_out is False else y_out), _ptr(workspace), workspace.numel(),
                            ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_f32(x, w, lut, stride, pad, x_range=None, w_range=None, relu=False, round_mode=0, acc_out=None, y_out=None,
                  workspace=None, stream=None):
    """Float layer.  x: float32 [N,H,W,Cin]; w: float32 [KH,KW,Cin,Cout]; ranges: float32 CUDA
    tensors of two, or None to let the layer take the range of that tensor.  Returns (acc_out, y_out); pass False to skip one of them."""
    L = lib()
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin,Cout]")
    d = _conv_desc(x.shape, w.shape, stride, pad)
    OH, OW = _out_hw(d)
    if OH <= 0 or OW <= 0:
        _check(-2)
    if _tune_arg() is not None:
        return _f32_ex(d, x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace, stream,
                       (d.N, OH, OW, d.Cout))
    acc_out, y_out = _outs((d.N, OH, OW, d.Cout), x.device, acc_out, y_out)
    if workspace is None:
        workspace = _workspace(ax_conv2d_f32_workspace_bytes(x.shape, w.shape, stride, pad), x.device, stream)
    _dev(workspace, torch.uint8, "workspace")
    rc = L.ax_conv2d_f32(_ptr(x), d.N, d.H, d.W, d.Cin, _ptr(w), d.KH, d.KW, d.Cout, _ptr(lut), d.stride_h, d.stride_w,
                         d.pad_h, d.pad_w, _ptr(x_range), _ptr(w_range), int(bool(relu)), int(round_mode),
                         _ptr(None if acc_out is False else acc_out), _ptr(None if y_out is False else y_out),
                         _ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr(stream)))
    _check(rc)
    return (None if acc_out is False else acc_out), (None if y_out is False else y_out)


def ax_conv2d_f32_ex(x, w, lut, stride, pad, x_range=None, w_range=None, relu=False, round_mode=0, dilation=1,
                     depthwise=False, signed=False, acc_out=None, y_out=None, workspace=None, stream=None, groups=1):
    """Float layer with dilation / signed codes / depthwise filters (w [KH,KW,Cin,mult]) / grouped
    filters (w [KH,KW,Cin/groups,Cout]).  Returns (acc_out, y_out); pass False to skip one of them."""
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 4 or w.dim() != 4 or w.shape[2] * int(groups) != x.shape[3]:
        raise ValueError("x must be [N,H,W,Cin] and w [KH,KW,Cin/groups,Cout] (or [KH,KW,Cin,mult])")
    desc = _conv_desc(x.shape, w.shape, stride, pad, dilation, depthwise, signed, groups)
    OH, OW = _out_hw(desc)
    if OH <= 0 or OW <= 0:
        _check(-2)
    return _f32_ex(desc, x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace, stream,
                   (desc.N, OH, OW, desc.Cout))


def ax_dense_f32(x, w, lut, x_range=None, w_range=None, relu=False, round_mode=0, acc_out=None, y_out=None, workspace=None,
                 stream=None):
    """x: float32 [M,K]; w: float32 [K,N]; outputs [M,N]."""
    L = lib()
    _f32_common(x, w, lut, x_range, w_range)
    if x.dim() != 2 or w.dim() != 2 or w.shape[0] != x.shape[1]:
        raise ValueError("x must be [M,K] and w [K,N]")
    M, K = x.shape
    N = w.shape[1]
    if _tune_arg() is not None:
        return _f32_ex(_dense_desc(M, K, N), x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace,
                       stream, (M, N))
    acc_out, y_out = _outs((M, N), x.device, acc_out, y_out)
    if workspace is None:
        workspace = _workspace(ax_dense_f32_workspace_bytes(M, K, N), x.device, stream)
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
