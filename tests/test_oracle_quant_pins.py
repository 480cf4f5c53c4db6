"""Pins of the float-layer oracle (range, coefficients, quantization, float-in / float-out
convolution) against things other than itself (CPU only): hand-computed cases, the invariants
Sec. II states (zero exactly representable, codes in [0, 255]), the half-step error bound of
rounding, library quantizers (torch's min/max observer, quantize_per_tensor and
fake_quantize_per_tensor_affine), a float64 convolution, and the already pinned integer oracle.
"""

import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I

import helpers as Hh

CASES = Hh.parse_cases(os.path.join(Hh.GOLDEN, "quant_cases.txt"))


def _f(s):
    return np.array(s.split(), dtype=np.float32)


def _i(s):
    return np.array(s.split(), dtype=np.int64)


@pytest.mark.parametrize("name", [n for n in CASES if n.startswith("Q")])
def test_hand_quantization_cases(name):
    c = CASES[name]
    for mode, key in ((0, "even"), (1, "away")):
        alpha, beta = oracle.coeffs(_f(c["range"]), mode)
        assert alpha == float(c["alpha"])
        assert beta == int(c["beta_" + key])
        codes = oracle.quantize_f32(_f(c["values"]), alpha, beta, relu=bool(int(c["relu"])), round_mode=mode)
        np.testing.assert_array_equal(codes.astype(np.int64), _i(c["codes_" + key]))


def test_hand_layer_case():
    c = CASES["L1"]
    x = _f(c["x"]).reshape([int(v) for v in c["x_shape"].split()])
    w = _f(c["w"]).reshape([int(v) for v in c["w_shape"].split()])
    r = oracle.conv2d_f32(x, w, I.lut_exact(), 1, 0, _f(c["x_range"]), _f(c["w_range"]))
    np.testing.assert_array_equal(r["xq"].reshape(-1).astype(np.int64), _i(c["xq"]))
    np.testing.assert_array_equal(r["wq"].reshape(-1).astype(np.int64), _i(c["wq"]))
    assert r["acc"].reshape(-1).tolist() == _i(c["acc"]).tolist()
    assert r["y"].reshape(-1).tolist() == _f(c["y"]).tolist()


def test_range_is_min_max():
    rng = np.random.default_rng(5)
    x = rng.standard_normal(100003).astype(np.float32) * 3
    r = oracle.range_f32(x)
    assert r[0] == x.min() and r[1] == x.max()
    r = oracle.range_f32(x, relu=True)
    assert r[0] == 0.0 and r[1] == x.max()
    r = oracle.range_f32(-np.abs(x) - 1, relu=True)  # all negative: ReLU leaves only zeros
    assert r[0] == 0.0 and r[1] == 0.0
    r = oracle.range_f32(np.array([4.25], np.float32))
    assert r[0] == 4.25 and r[1] == 4.25


RANGES = [(-1.0, 1.0), (0.0, 6.0), (-0.37, 0.41), (0.5, 3.0), (-5.0, -1.0), (-1e-3, 2e3), (-7.7, 0.0)]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("lohi", RANGES)
def test_zero_is_exactly_representable_and_codes_span(lohi, mode):
    alpha, beta = oracle.coeffs(np.array(lohi, np.float32), mode)
    assert alpha > 0 and 0 <= beta <= 255
    lo, hi = min(lohi[0], 0.0), max(lohi[1], 0.0)
    pts = np.array([0.0, -0.0, lo, hi], np.float32)
    codes = oracle.quantize_f32(pts, alpha, beta, round_mode=mode).astype(int)
    assert codes[0] == beta and codes[1] == beta  # r = 0 <-> code beta, and alpha * (beta - beta) = 0
    assert codes[2] == 0  # round(lo/alpha) = -round(-lo/alpha) = -beta for both modes
    assert codes[3] >= 254  # the top of the range reaches the last code (up to the rounding of beta)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("lohi", RANGES)
def test_rounding_error_at_most_half_a_step_and_monotone(lohi, mode):
    rng = np.random.default_rng(11)
    lo, hi = min(lohi[0], 0.0), max(lohi[1], 0.0)
    r = np.sort((rng.random(20000) * (hi - lo) + lo).astype(np.float32))
    alpha, beta = oracle.coeffs(np.array(lohi, np.float32), mode)
    codes = oracle.quantize_f32(r, alpha, beta, round_mode=mode).astype(np.float64)
    assert np.all(np.diff(codes) >= 0)
    back = np.float64(alpha) * (codes - beta)
    # Interior codes are within half a step; at the two ends the clamp can add the rounding of beta.
    interior = (codes > 0) & (codes < 255)
    # (the float32 quotient r/alpha, up to 255, carries a rounding error of about 1e-5 steps)
    assert np.all(np.abs(back - r)[interior] <= 0.5 * alpha * (1 + 2e-4))
    assert np.all(np.abs(back - r) <= 1.0 * alpha * (1 + 2e-4))


@pytest.mark.parametrize("lohi", RANGES)
def test_coefficients_match_library_observer(lohi):
    obs = torch.ao.quantization.observer.MinMaxObserver(dtype=torch.quint8, qscheme=torch.per_tensor_affine)
    obs(torch.tensor(lohi, dtype=torch.float32))
    scale, zp = obs.calculate_qparams()
    alpha, beta = oracle.coeffs(np.array(lohi, np.float32), 0)
    assert abs(alpha - float(scale)) <= 1e-6 * alpha
    # The observer rounds min/scale with its own tie rule; away from ties the zero point is the same.
    frac = (-min(lohi[0], 0.0) / alpha) % 1.0
    if abs(frac - 0.5) > 1e-3:
        assert beta == int(zp)


@pytest.mark.parametrize("dist", ["normal", "relu", "uniform"])
def test_codes_match_library_quantizer(dist):
    rng = np.random.default_rng(21)
    x = rng.standard_normal(200000).astype(np.float32)
    if dist == "relu":
        x = np.maximum(x, 0)
    if dist == "uniform":
        x = (rng.random(200000) * 12 - 3).astype(np.float32)
    alpha, beta = oracle.coeffs(oracle.range_f32(x), 0)
    codes = oracle.quantize_f32(x, alpha, beta).astype(np.int64)
    lib = torch.quantize_per_tensor(torch.from_numpy(x), alpha, beta, torch.quint8).int_repr().numpy().astype(np.int64)
    diff = np.abs(codes - lib)
    # The library multiplies by 1/alpha where the oracle divides: codes may differ by one only
    # where the quotient is within float rounding of a tie.
    assert diff.max() <= 1
    assert (diff != 0).mean() < 1e-4
    q64 = np.float64(x) / np.float64(alpha)
    tie = np.abs((q64 % 1.0) - 0.5) < 1e-4
    np.testing.assert_array_equal(codes[~tie], lib[~tie])
    # and against plain float64 arithmetic
    ref = np.clip(np.rint(q64) + beta, 0, 255).astype(np.int64)
    np.testing.assert_array_equal(codes[~tie], ref[~tie])


def test_round_modes_differ_only_at_ties():
    rng = np.random.default_rng(22)
    x = (rng.integers(-300, 300, 5000) * 0.5).astype(np.float32)  # every other value is a tie for alpha = 1
    even = oracle.quantize_f32(x, 1.0, 100, round_mode=0).astype(int)
    away = oracle.quantize_f32(x, 1.0, 100, round_mode=1).astype(int)
    ref_even = np.clip(np.rint(x.astype(np.float64)) + 100, 0, 255)
    ref_away = np.clip(np.sign(x) * np.floor(np.abs(x.astype(np.float64)) + 0.5) + 100, 0, 255)
    np.testing.assert_array_equal(even, ref_even.astype(int))
    np.testing.assert_array_equal(away, ref_away.astype(int))
    assert (even != away).any()


LAYERS = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad
    (2, 9, 8, 5, 3, 3, 6, 1, 1),
    (1, 10, 10, 8, 1, 1, 12, 2, 0),
    (2, 7, 7, 3, 5, 5, 4, 2, 2),
]


def _float_layer(shape, seed):
    N, H, W, Cin, KH, KW, Cout, s, p = shape
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    w = (rng.standard_normal((KH, KW, Cin, Cout)) * 0.2).astype(np.float32)
    return x, w, s, p


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", LAYERS)
def test_float_layer_composes_pinned_parts(shape, relu):
    """The float layer's integer part must be the (separately pinned) integer oracle applied to
    its own codes, and its float output the same product computed in double."""
    x, w, s, p = _float_layer(shape, 31)
    xr, wr = oracle.range_f32(x, relu), oracle.range_f32(w)
    lut = I.lut_random_error(7)
    r = oracle.conv2d_f32(x, w, lut, s, p, xr, wr, relu=relu)
    q = I.Quant(r["x_scale"], r["x_zp"], r["w_scale"], r["w_zp"], -1)
    acc, y = oracle.conv2d(r["xq"], r["wq"], lut, s, p, q)
    np.testing.assert_array_equal(r["acc"], acc)
    assert Hh.float_ok(r["y"], y, rtol=2e-7, atol=1e-30)  # one float32 product vs one rounded double product
    np.testing.assert_array_equal(r["xq"], oracle.quantize_f32(np.maximum(x, 0) if relu else x, r["x_scale"], r["x_zp"]))


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", LAYERS)
def test_float_layer_with_exact_table_equals_fake_quantized_convolution(shape, relu):
    """With the exact multiplier the layer equals a real-valued convolution of the two
    quantize-dequantize'd tensors (the paper's accuracy statement for the exact table), here
    with the library's fake quantizer and a float64 convolution."""
    x, w, s, p = _float_layer(shape, 32)
    xr, wr = oracle.range_f32(x, relu), oracle.range_f32(w)
    r = oracle.conv2d_f32(x, w, I.lut_exact(), s, p, xr, wr, relu=relu)
    xt = torch.from_numpy(np.maximum(x, 0) if relu else x)
    xf = torch.fake_quantize_per_tensor_affine(xt, r["x_scale"], r["x_zp"], 0, 255).double()
    wf = torch.fake_quantize_per_tensor_affine(torch.from_numpy(w), r["w_scale"], r["w_zp"], 0, 255).double()
    ref = torch.nn.functional.conv2d(xf.permute(0, 3, 1, 2), wf.permute(3, 2, 0, 1), stride=s, padding=p)
    ref = ref.permute(0, 2, 3, 1).numpy()
    # a handful of codes may differ by one at float ties (see test_codes_match_library_quantizer):
    # compare with a tolerance of a few quantization steps' products instead of 1e-5
    step = r["x_scale"] * np.abs(wf.numpy()).max() + r["w_scale"] * np.abs(xf.numpy()).max()
    close = np.abs(r["y"] - ref) <= 1e-5 * np.abs(ref) + 1e-5
    assert close.mean() > 0.99
    assert np.abs(r["y"] - ref).max() <= 2 * step


@pytest.mark.parametrize("shape", LAYERS)
def test_float_layer_close_to_unquantized_convolution(shape):
    """Quantization error bound: each operand is off by at most half a step, so every output
    differs from the float64 convolution of the raw tensors by at most
    sum_k (|x| * aw/2 + |w| * ax/2 + ax*aw/4)."""
    x, w, s, p = _float_layer(shape, 33)
    r = oracle.conv2d_f32(x, w, I.lut_exact(), s, p, oracle.range_f32(x), oracle.range_f32(w))
    xd, wd = torch.from_numpy(x).double(), torch.from_numpy(w).double()

    def conv(a, b):
        return torch.nn.functional.conv2d(a.permute(0, 3, 1, 2), b.permute(3, 2, 0, 1), stride=s,
                                          padding=p).permute(0, 2, 3, 1).numpy()

    ref = conv(xd, wd)
    ax, aw = r["x_scale"], r["w_scale"]
    bound = conv(xd.abs(), torch.full_like(wd, aw / 2)) + conv(torch.full_like(xd, ax / 2), wd.abs()) \
        + conv(torch.full_like(xd, ax / 2), torch.full_like(wd, aw / 2))
    assert np.all(np.abs(r["y"] - ref) <= bound * (1 + 1e-4) + 1e-5)
    assert np.abs(r["y"] - ref).max() > 0  # it is a quantized result, not the float one


# ---- the float layer with the full parameter set (dilation, signed codes, depthwise) --------------

EX_CASES = [
    # N, H, W, Cin, KH, KW, last, stride, pad, dilation, depthwise   (last = Cout, or the multiplier)
    (2, 9, 8, 5, 3, 3, 6, 1, 2, 2, False),
    (1, 10, 10, 4, 3, 2, 3, 2, 3, (3, 2), False),
    (2, 8, 8, 6, 3, 3, 2, 1, 1, 1, True),
    (1, 9, 9, 3, 3, 3, 1, 2, 2, 2, True),
]


def _ex_operands(case, seed):
    N, H, W, Cin, KH, KW, last, s, p, d, dwise = case
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    w = (rng.standard_normal((KH, KW, Cin, last)) * 0.2).astype(np.float32)
    return x, w, s, p, d, dwise


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", EX_CASES)
def test_extended_float_layer_composes_pinned_parts(case, signed):
    """Its integer part must be the (separately pinned) variant oracle applied to its own codes and
    coefficients, its codes the pinned quantization (lowered by 128 when signed)."""
    x, w, s, p, d, dwise = _ex_operands(case, 41)
    relu = not signed
    xr, wr = oracle.range_f32(x, relu), oracle.range_f32(w)
    lut = I.lut_signed_random_error(9) if signed else I.lut_random_error(9)
    r = oracle.conv2d_f32_ex(x, w, lut, s, p, xr, wr, relu=relu, dilation=d, depthwise=dwise, signed=signed)
    au, bu = oracle.coeffs(xr)
    codes_u = oracle.quantize_f32(x, au, bu, relu=relu).astype(np.int64)
    np.testing.assert_array_equal(r["xq"].astype(np.int64), codes_u - (128 if signed else 0))
    assert r["x_zp"] == bu - (128 if signed else 0) and r["x_scale"] == au
    q = I.Quant(r["x_scale"], r["x_zp"], r["w_scale"], r["w_zp"], None)
    acc, y = oracle.conv2d_ex(r["xq"], r["wq"], lut, s, p, q, dilation=d, depthwise=dwise, signed=signed)
    np.testing.assert_array_equal(r["acc"], acc)
    assert Hh.float_ok(r["y"], y, rtol=2e-7, atol=1e-30)


@pytest.mark.parametrize("case", EX_CASES)
def test_signed_and_unsigned_float_layers_agree_with_exact_multipliers(case):
    """(a - beta1)(b - beta2) does not change when codes and zero points are lowered by 128: with
    the exact signed and the exact unsigned multiplier the two forms give the same outputs."""
    x, w, s, p, d, dwise = _ex_operands(case, 42)
    xr, wr = oracle.range_f32(x), oracle.range_f32(w)
    ru = oracle.conv2d_f32_ex(x, w, I.lut_exact(), s, p, xr, wr, dilation=d, depthwise=dwise)
    rs = oracle.conv2d_f32_ex(x, w, I.lut_signed_exact(), s, p, xr, wr, dilation=d, depthwise=dwise, signed=True)
    np.testing.assert_array_equal(ru["y"], rs["y"])
    assert (ru["acc"] != rs["acc"]).any()  # the raw sums differ, only the corrected result is the same


@pytest.mark.parametrize("case", EX_CASES)
def test_extended_float_layer_exact_table_equals_library_convolution(case):
    N, H, W, Cin, KH, KW, last, s, p, d, dwise = case
    x, w, s, p, d, dwise = _ex_operands(case, 43)
    r = oracle.conv2d_f32_ex(x, w, I.lut_signed_exact(), s, p, oracle.range_f32(x), oracle.range_f32(w), dilation=d,
                             depthwise=dwise, signed=True)
    xf = r["x_scale"] * (torch.from_numpy(r["xq"].astype(np.float64)) - r["x_zp"])
    wf = r["w_scale"] * (torch.from_numpy(r["wq"].astype(np.float64)) - r["w_zp"])
    pair = lambda v: (v, v) if np.isscalar(v) else tuple(v)
    if dwise:
        wt = wf.permute(2, 3, 0, 1).reshape(Cin * last, 1, KH, KW)
        ref = torch.nn.functional.conv2d(xf.permute(0, 3, 1, 2), wt, stride=pair(s), padding=pair(p), dilation=pair(d),
                                         groups=Cin)
    else:
        ref = torch.nn.functional.conv2d(xf.permute(0, 3, 1, 2), wf.permute(3, 2, 0, 1), stride=pair(s),
                                         padding=pair(p), dilation=pair(d))
    assert Hh.float_ok(r["y"], ref.permute(0, 2, 3, 1).numpy(), rtol=1e-5, atol=1e-5)
    # and it is a quantization of the unquantized convolution: zero real input stays exactly zero
    z = oracle.conv2d_f32_ex(np.zeros_like(x), w, I.lut_signed_exact(), s, p, oracle.range_f32(x), oracle.range_f32(w),
                             dilation=d, depthwise=dwise, signed=True)
    assert not z["y"].any()
