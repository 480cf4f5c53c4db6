"""Seeded synthetic inputs: multiplier tables, quantized tensors and layer shape lists.

This module feeds both the CPU oracle and the HIP library.  It contains no part of the
method itself (no lookup, no accumulation, no correction terms): it only produces the
operands -- ``uint8`` activation and filter codes, affine quantization parameters
(scale, zero point; Eq. (1) of the paper, Sec. II) and 256x256 ``uint16`` multiplier
truth tables (Sec. II: a table of 256^2 16-bit products, 128 kB).

The paper evaluated CIFAR-10 images on pre-trained ResNets; neither is available, so the
tensors below reproduce shapes and value distributions only (uniform codes, clipped-ReLU
and Gaussian tensors quantized per tensor from their min/max).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

# ----------------------------------------------------------------------------------------
# multiplier truth tables, all indexed lut[a * 256 + b], a = activation code, b = filter code
# ----------------------------------------------------------------------------------------


def _grid() -> Tuple[np.ndarray, np.ndarray]:
    a = np.arange(256, dtype=np.int64).reshape(256, 1)
    b = np.arange(256, dtype=np.int64).reshape(1, 256)
    return a, b


def lut_exact() -> np.ndarray:
    """Exact 8x8-bit unsigned multiplier: entry (a, b) holds a*b."""
    a, b = _grid()
    return (a * b).astype(np.uint16).reshape(-1)


def lut_truncated(t: int) -> np.ndarray:
    """Array multiplier with the partial-product bits of weight below 2**t removed.

    Entry (a, b) is the sum of a_i * b_j * 2**(i+j) over bit pairs with i + j >= t, so the
    carries those bits would have produced vanish as well (this differs from masking the
    low bits of the exact product).  t = 0 gives the exact table.
    """
    if not 0 <= t <= 15:
        raise ValueError("t must be in [0, 15]")
    a, b = _grid()
    acc = np.zeros((256, 256), dtype=np.int64)
    for i in range(8):
        for j in range(8):
            if i + j >= t:
                acc += (((a >> i) & 1) * ((b >> j) & 1)) << (i + j)
    return acc.astype(np.uint16).reshape(-1)


def lut_random_error(seed: int, amplitude: int = 64) -> np.ndarray:
    """Exact product plus an i.i.d. uniform integer error in [-amplitude, amplitude] on every
    entry (zero operands included), clamped to the uint16 range."""
    rng = np.random.default_rng(seed)
    a, b = _grid()
    err = rng.integers(-amplitude, amplitude + 1, size=(256, 256), dtype=np.int64)
    return np.clip(a * b + err, 0, 65535).astype(np.uint16).reshape(-1)


def lut_zero() -> np.ndarray:
    return np.zeros(65536, dtype=np.uint16)


def lut_const(c: int) -> np.ndarray:
    return np.full(65536, c, dtype=np.uint16)


def lut_onehot(a0: int, b0: int, value: int = 1) -> np.ndarray:
    t = np.zeros((256, 256), dtype=np.uint16)
    t[a0, b0] = value
    return t.reshape(-1)


def lut_first_operand() -> np.ndarray:
    """Entry (a, b) = a: a deliberately non-commutative table."""
    a, b = _grid()
    return (a + 0 * b).astype(np.uint16).reshape(-1)


def lut_second_operand() -> np.ndarray:
    """Entry (a, b) = b."""
    a, b = _grid()
    return (0 * a + b).astype(np.uint16).reshape(-1)


def lut_signed_exact() -> np.ndarray:
    """Signed 8x8 multiplier as int16 [256,256], addressed by the operands' two's-complement
    bit patterns: entry [a & 255][b & 255] = a * b for a, b in [-128, 127]."""
    p = np.arange(256, dtype=np.int64)
    v = np.where(p < 128, p, p - 256)
    return (v[:, None] * v[None, :]).astype(np.int16)


def lut_signed_random_error(seed: int, amplitude: int = 64) -> np.ndarray:
    """Signed exact product plus a uniform integer error in [-amplitude, amplitude] on every
    entry, clipped to int16."""
    rng = np.random.default_rng(seed)
    err = rng.integers(-amplitude, amplitude + 1, size=(256, 256), dtype=np.int64)
    return np.clip(lut_signed_exact().astype(np.int64) + err, -32768, 32767).astype(np.int16)


def lut_signed_random(seed: int) -> np.ndarray:
    """Arbitrary int16 entries over the whole range (stress: sums of either sign)."""
    rng = np.random.default_rng(seed)
    return rng.integers(-32768, 32768, size=(256, 256), dtype=np.int64).astype(np.int16)


def lut_random(seed: int) -> np.ndarray:
    """Every entry an independent uniform uint16: no multiplier structure at all."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, 65536, size=65536, dtype=np.int64).astype(np.uint16)


# ----------------------------------------------------------------------------------------
# affine quantization of synthetic real tensors (scale alpha, zero point beta; Eq. (1))
# ----------------------------------------------------------------------------------------


@dataclass
class Quant:
    """Quantization parameters handed to a layer call.

    x_scale/x_zp are alpha_1/beta_1 and w_scale/w_zp are alpha_2/beta_2 of Eq. (3).
    pad_code is the activation code fed to the multiplier for taps outside the image
    (-1: use x_zp, the code of the real value zero).
    """

    x_scale: float = 1.0
    x_zp: int = 0
    w_scale: float = 1.0
    w_zp: int = 0
    pad_code: int = -1


def quantize_per_tensor(r: np.ndarray) -> Tuple[np.ndarray, float, int]:
    """Map a real tensor to uint8 codes from its own min/max so that r ~ scale*(code - zp)
    and the real value 0 is exactly representable.  Rounding is half-to-even."""
    r = np.asarray(r, dtype=np.float64)
    lo = min(float(r.min()), 0.0)
    hi = max(float(r.max()), 0.0)
    scale = (hi - lo) / 255.0
    if scale == 0.0:
        scale = 1.0
    zp = int(np.clip(np.rint(-lo / scale), 0, 255))
    codes = np.clip(np.rint(r / scale) + zp, 0, 255).astype(np.uint8)
    return codes, float(np.float32(scale)), zp


# ----------------------------------------------------------------------------------------
# layer descriptions
# ----------------------------------------------------------------------------------------


@dataclass
class Layer:
    """One conv2d (NHWC input, HWIO filters) or dense (H = W = KH = KW = 1) call."""

    name: str
    N: int
    H: int
    W: int
    Cin: int
    KH: int
    KW: int
    Cout: int
    stride: int = 1
    pad: int = 0
    dense: bool = False
    x_dist: str = "uniform"  # uniform | relu | relu6 | normal
    w_dist: str = "uniform"  # uniform | normal | normal01
    count: int = 1  # how many times this shape occurs in the network

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1

    @property
    def M(self) -> int:
        return self.N * self.OH * self.OW

    @property
    def K(self) -> int:
        return self.KH * self.KW * self.Cin

    @property
    def macs(self) -> int:
        """Lookups of one call, padded taps included."""
        return self.M * self.K * self.Cout

    @property
    def algorithmic_bytes(self) -> int:
        """Each operand read once, the table once, both outputs written once."""
        return self.N * self.H * self.W * self.Cin + self.K * self.Cout + 131072 + 8 * self.M * self.Cout


def make_operands(layer: Layer, seed: int) -> Tuple[np.ndarray, np.ndarray, Quant]:
    """Activation codes (N,H,W,Cin), filter codes (KH,KW,Cin,Cout) and their parameters."""
    rng = np.random.default_rng(seed)
    xs = (layer.N, layer.H, layer.W, layer.Cin)
    ws = (layer.KH, layer.KW, layer.Cin, layer.Cout)
    q = Quant()
    if layer.x_dist == "uniform":
        x = rng.integers(0, 256, size=xs, dtype=np.int64).astype(np.uint8)
        q.x_scale, q.x_zp = 1.0 / 64.0, 128
    else:
        r = rng.standard_normal(size=xs, dtype=np.float32)
        if layer.x_dist == "relu":
            np.maximum(r, 0.0, out=r)
        elif layer.x_dist == "relu6":
            np.clip(r, 0.0, 6.0, out=r)
        elif layer.x_dist != "normal":
            raise ValueError(layer.x_dist)
        x, q.x_scale, q.x_zp = quantize_per_tensor(r)
    if layer.w_dist == "uniform":
        w = rng.integers(0, 256, size=ws, dtype=np.int64).astype(np.uint8)
        q.w_scale, q.w_zp = 1.0 / 128.0, 128
    else:
        sigma = {"normal": 1.0, "normal01": 0.1}[layer.w_dist]
        r = rng.standard_normal(size=ws, dtype=np.float32) * np.float32(sigma)
        w, q.w_scale, q.w_zp = quantize_per_tensor(r)
    q.pad_code = -1
    return x, w, q


def make_float_operands(layer: Layer, seed: int):
    """Real-valued activations (N,H,W,Cin) and filters (KH,KW,Cin,Cout) as float32, for the
    float-in / float-out form of the layer.  Activations are standard normal (the layer's own
    ReLU option, not the generator, clips them); "uniform" layers draw from [-2, 2).  Filters
    are normal with the layer's sigma, or uniform in [-1, 1)."""
    rng = np.random.default_rng(seed)
    xs = (layer.N, layer.H, layer.W, layer.Cin)
    ws = (layer.KH, layer.KW, layer.Cin, layer.Cout)
    if layer.x_dist == "uniform":
        x = (rng.random(size=xs, dtype=np.float32) * np.float32(4.0) - np.float32(2.0)).astype(np.float32)
    else:
        x = rng.standard_normal(size=xs, dtype=np.float32)
        if layer.x_dist == "relu6":
            np.minimum(x, 6.0, out=x)
    if layer.w_dist == "uniform":
        w = (rng.random(size=ws, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    else:
        sigma = {"normal": 1.0, "normal01": 0.1}[layer.w_dist]
        w = rng.standard_normal(size=ws, dtype=np.float32) * np.float32(sigma)
    return x, w


# ----------------------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------------------


def config_single_layer() -> List[Layer]:
    """One small 3x3 layer on uniform codes (run with the t=4 truncated and the exact table)."""
    return [Layer("c1.conv3x3", 1, 16, 16, 8, 3, 3, 8, 1, 1)]


def config_resnet8_cifar(batch: int = 128) -> List[Layer]:
    """CIFAR-shaped residual stack: seven 3x3 pad-1 layers, widths 16/32/64."""
    L = []
    L.append(Layer("c2.l0", batch, 32, 32, 3, 3, 3, 16, 1, 1, x_dist="normal", w_dist="normal01"))
    L.append(Layer("c2.l1", batch, 32, 32, 16, 3, 3, 16, 1, 1, x_dist="relu6", w_dist="normal01"))
    L.append(Layer("c2.l2", batch, 32, 32, 16, 3, 3, 16, 1, 1, x_dist="relu6", w_dist="normal01"))
    L.append(Layer("c2.l3", batch, 32, 32, 16, 3, 3, 32, 2, 1, x_dist="relu6", w_dist="normal01"))
    L.append(Layer("c2.l4", batch, 16, 16, 32, 3, 3, 32, 1, 1, x_dist="relu6", w_dist="normal01"))
    L.append(Layer("c2.l5", batch, 16, 16, 32, 3, 3, 64, 2, 1, x_dist="relu6", w_dist="normal01"))
    L.append(Layer("c2.l6", batch, 8, 8, 64, 3, 3, 64, 1, 1, x_dist="relu6", w_dist="normal01"))
    return L


def config_resnet50(batch: int = 32, unique: bool = False) -> List[Layer]:
    """All 53 convolutions of an ImageNet-shaped ResNet-50 (stride on the 3x3 of each
    down-sampling block) followed by the 2048x1000 classifier as a dense call.

    With ``unique`` the repeated shapes are merged and ``count`` says how often each occurs.
    """
    L: List[Layer] = []

    def conv(name, hw, cin, k, cout, s=1, p=0, x_dist="relu"):
        L.append(Layer(name, batch, hw, hw, cin, k, k, cout, s, p, x_dist=x_dist, w_dist="normal"))

    conv("conv1", 224, 3, 7, 64, 2, 3, x_dist="uniform")
    hw, cin = 56, 64
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=1):
        out = 4 * mid
        for b in range(blocks):
            s = 2 if (b == 0 and stage > 1) else 1
            tag = "s%db%d" % (stage, b)
            conv(tag + ".a1x1", hw, cin, 1, mid)
            conv(tag + ".b3x3", hw, mid, 3, mid, s, 1)
            if b == 0:
                conv(tag + ".proj", hw, cin, 1, out, s, 0)
            hw = hw // s
            conv(tag + ".c1x1", hw, mid, 1, out)
            cin = out
    L.append(Layer("fc", batch, 1, 1, 2048, 1, 1, 1000, dense=True, x_dist="relu", w_dist="normal"))
    if not unique:
        return L
    merged: List[Layer] = []
    for l in L:
        for m in merged:
            if (m.H, m.Cin, m.KH, m.Cout, m.stride, m.dense) == (l.H, l.Cin, l.KH, l.Cout, l.stride, l.dense):
                m.count += 1
                break
        else:
            merged.append(Layer(**{**l.__dict__}))
    return merged


def config_lut_sweep(batch: int = 64) -> List[Layer]:
    """Two stage-3-like layers evaluated against many tables back to back."""
    return [
        Layer("c4.A1x1", batch, 28, 28, 512, 1, 1, 128),
        Layer("c4.B3x3", batch, 28, 28, 128, 3, 3, 128, 1, 1),
    ]


def config_gemm_shaped() -> List[Layer]:
    """Large-channel 1x1 convolution and a square dense layer."""
    return [
        Layer("c5.conv1x1", 16, 14, 14, 1024, 1, 1, 2048),
        Layer("c5.fc", 256, 1, 1, 4096, 1, 1, 4096, dense=True),
    ]


def layer_seed(config: int, index: int) -> int:
    """Seed rule shared by tests and the benchmark: config 1 uses seed 0."""
    return 0 if config == 1 else 1000 * config + index
