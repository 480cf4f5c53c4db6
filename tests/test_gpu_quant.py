"""GPU parity of the float side of the layer (range, coefficients, quantization, the float-in /
float-out convolution and a chained run), through the C ABI, against the CPU oracle on the same
seeded float tensors.  Ranges, coefficients, codes and int32 accumulators: bit exact.  Float
outputs: within 1e-5 relative + 1e-6 absolute (and, since both sides apply the same float32
operations in the same order, in practice identical)."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    ax.ax_set_option("variant", 0)
    ax.ax_set_option("split_k", 0)
    ax.ax_set_option("tile", 0)
    ax.ax_set_option("row_tiles", 0)


def _data(n, seed, kind="normal"):
    rng = np.random.default_rng(seed)
    if kind == "normal":
        return (rng.standard_normal(n) * 2.5).astype(np.float32)
    if kind == "positive":
        return (rng.random(n) * 6 + 0.25).astype(np.float32)
    if kind == "negative":
        return (-rng.random(n) * 3 - 0.5).astype(np.float32)
    if kind == "ties":  # multiples of one half: every other quotient is a tie when alpha = 1
        return (rng.integers(-256, 255, n) * 0.5).astype(np.float32)
    raise ValueError(kind)


SIZES = [1, 2, 3, 4, 5, 63, 64, 255, 1024, 4099, 1000003, 6 * 1024 * 1024 + 7]


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("n", SIZES)
def test_range_matches_oracle(n, relu):
    for kind in ("normal", "positive", "negative"):
        x = _data(n, n % 1000 + 3, kind)
        got = ax.ax_range_f32(G.to_dev(x), relu=relu).cpu().numpy()
        want = oracle.range_f32(x, relu=relu)
        assert got[0] == want[0] and got[1] == want[1], (kind, got, want)


@pytest.mark.parametrize("offset", [1, 2, 3])
def test_range_and_codes_on_unaligned_views(offset):
    x = _data(70001, 9)
    xd = G.to_dev(x)
    view = xd[offset:]
    got = ax.ax_range_f32(view).cpu().numpy()
    want = oracle.range_f32(x[offset:])
    assert got[0] == want[0] and got[1] == want[1]
    rng = G.to_dev(want)
    out = torch.zeros(x.size + 8, dtype=torch.uint8, device="cuda")
    for oofs in (0, 1, 2, 3):  # output start aligned to 4 bytes or not
        codes, co = ax.ax_quantize_f32(view, rng, codes_out=out[oofs:oofs + view.numel()])
        alpha, beta = oracle.coeffs(want)
        np.testing.assert_array_equal(codes.cpu().numpy(), oracle.quantize_f32(x[offset:], alpha, beta))


def _coeffs_of(co):
    c = co.cpu().numpy()
    return float(c[:1].view(np.float32)[0]), int(c[1])


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("kind", ["normal", "positive", "negative", "ties"])
@pytest.mark.parametrize("n", [1, 7, 64, 4099, 1000003])
def test_quantize_matches_oracle(n, kind, relu, mode):
    x = _data(n, n % 977 + 11, kind)
    want_range = oracle.range_f32(x, relu=relu)
    if kind == "ties":
        want_range = np.array([-128.0, 127.0], np.float32)  # alpha = 1: quotients are the values themselves
    codes, co = ax.ax_quantize_f32(G.to_dev(x), G.to_dev(want_range), relu=relu, round_mode=mode)
    alpha, beta = oracle.coeffs(want_range, mode)
    ga, gb = _coeffs_of(co)
    assert ga == alpha and gb == beta
    np.testing.assert_array_equal(codes.cpu().numpy(), oracle.quantize_f32(x, alpha, beta, relu=relu, round_mode=mode))


@pytest.mark.parametrize("lohi", [(-0.5, 0.5), (0.0, 0.0), (1.0, 2.0), (-3.0, -1.0), (-1.0, 509.0), (0.0, 1e-30)])
def test_quantize_saturates_outside_a_given_range(lohi):
    x = _data(50001, 4)
    rng = np.array(lohi, np.float32)
    for mode in (0, 1):
        codes, co = ax.ax_quantize_f32(G.to_dev(x), G.to_dev(rng), round_mode=mode)
        alpha, beta = oracle.coeffs(rng, mode)
        assert _coeffs_of(co) == (alpha, beta)
        np.testing.assert_array_equal(codes.cpu().numpy(), oracle.quantize_f32(x, alpha, beta, round_mode=mode))


def L(N, H, W, Cin, KH, KW, Cout, s=1, p=0, dense=False, x_dist="normal", w_dist="normal01"):
    return I.Layer("f%dx%dx%dx%d_k%dx%d_c%d_s%d_p%d" % (N, H, W, Cin, KH, KW, Cout, s, p),
                   N, H, W, Cin, KH, KW, Cout, s, p, dense=dense, x_dist=x_dist, w_dist=w_dist)


def _run_f32(layer, seed, lut, relu, mode, x=None, w=None, given="xw"):
    """given: which ranges are handed to the layer ("xw", "x", "w" or ""); the layer takes the
    others itself."""
    if x is None:
        x, w = I.make_float_operands(layer, seed)
    xd, wd, ld = G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut)
    xr = ax.ax_range_f32(xd, relu=relu) if "x" in given else None
    wr = ax.ax_range_f32(wd) if "w" in given else None
    if layer.dense:
        acc, y = ax.ax_dense_f32(xd.view(x.shape[0], -1), wd.view(-1, w.shape[-1]), ld, xr, wr, relu=relu,
                                 round_mode=mode)
    else:
        acc, y = ax.ax_conv2d_f32(xd, wd, ld, layer.stride, layer.pad, xr, wr, relu=relu, round_mode=mode)
    torch.cuda.synchronize()
    ref = oracle.conv2d_f32(x, w, lut, layer.stride, layer.pad, oracle.range_f32(x, relu), oracle.range_f32(w),
                            relu=relu, round_mode=mode)
    return acc.cpu().numpy(), y.cpu().numpy(), ref


def _check_f32(layer, seed, lut, relu=False, mode=0, given="xw"):
    acc, y, ref = _run_f32(layer, seed, lut, relu, mode, given=given)
    G.assert_parity(acc, y, ref["acc"], ref["y"], layer.name)
    np.testing.assert_array_equal(y.reshape(-1), ref["y"].reshape(-1))
    return ref


FLOAT_LAYERS = [
    L(1, 1, 1, 1, 1, 1, 1),
    L(2, 9, 7, 5, 3, 3, 6, 2, 1),
    L(1, 4, 4, 2, 3, 3, 2, 1, 3),                 # padding wider than the kernel
    L(1, 40, 40, 16, 3, 3, 72, 1, 1),
    L(2, 30, 30, 20, 5, 5, 9, 2, 2),              # Cin not a multiple of 16: materialized patches
    L(1, 64, 64, 3, 7, 7, 16, 2, 3),              # stem-like
    L(2, 14, 14, 256, 1, 1, 520, 1, 0),           # ragged channel tile
    L(1, 7, 7, 512, 3, 3, 512, 1, 1),             # few pixels, many channels
    L(64, 1, 1, 512, 1, 1, 100, dense=True),
    L(3, 1, 1, 37, 1, 1, 11, dense=True),
]


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("layer", FLOAT_LAYERS, ids=lambda l: l.name)
def test_float_layer_matches_oracle(layer, variant):
    ax.ax_set_option("variant", variant)
    lut = I.lut_random_error(77)
    relu = (layer.Cin % 2 == 0)
    _check_f32(layer, 500 + layer.Cout, lut, relu=relu, mode=variant & 1)


@pytest.mark.parametrize("given", ["", "x", "w"])
@pytest.mark.parametrize("layer", FLOAT_LAYERS, ids=lambda l: l.name)
def test_float_layer_takes_missing_ranges_itself(layer, given):
    relu = (layer.Cin % 2 == 1)
    _check_f32(layer, 700 + layer.Cout, I.lut_random_error(78), relu=relu, mode=len(given), given=given)


@pytest.mark.parametrize("split", [2, 3])
def test_float_layer_with_forced_k_split(split):
    ax.ax_set_option("split_k", split)
    _check_f32(L(1, 20, 20, 64, 3, 3, 64, 1, 1), 41, I.lut_truncated(5), relu=True)


def test_float_layer_zero_point_of_shifted_activations():
    """Activations that are all positive or all negative still widen the range to zero; the pad
    code is then 0 or 255 and must reach the table through the device-side coefficients."""
    lut = I.lut_random_error(5)
    for shift in (3.0, -3.0):
        layer = L(2, 12, 12, 16, 3, 3, 24, 1, 1)
        x, w = I.make_float_operands(layer, 8)
        x = (np.abs(x) * np.float32(np.sign(shift)) + np.float32(shift)).astype(np.float32)
        acc, y, ref = _run_f32(layer, 0, lut, False, 0, x=x, w=w)
        assert ref["x_zp"] == (0 if shift > 0 else 255)
        G.assert_parity(acc, y, ref["acc"], ref["y"], "shift %g" % shift)


def test_float_layer_exact_table_is_close_to_float_convolution():
    """End-to-end sanity on the device path alone: with the exact multiplier the layer is a
    quantized convolution, within the half-step error bound of the float64 result."""
    layer = L(2, 16, 16, 32, 3, 3, 48, 1, 1)
    x, w = I.make_float_operands(layer, 12)
    acc, y, ref = _run_f32(layer, 0, I.lut_exact(), False, 0, x=x, w=w)
    xd, wd = torch.from_numpy(x).double(), torch.from_numpy(w).double()
    full = torch.nn.functional.conv2d(xd.permute(0, 3, 1, 2), wd.permute(3, 2, 0, 1), padding=1).permute(0, 2, 3, 1)
    ax_, aw_ = ref["x_scale"], ref["w_scale"]
    K = layer.K
    bound = K * (np.abs(x).max() * aw_ / 2 + np.abs(w).max() * ax_ / 2 + ax_ * aw_ / 4)
    assert np.abs(y - full.numpy()).max() <= bound
    assert np.corrcoef(y.reshape(-1), full.numpy().reshape(-1))[0, 1] > 0.999


def test_chained_stack_matches_oracle_layer_by_layer():
    """Seven chained 3x3 layers (the CIFAR-sized stack): each layer's float output, after ReLU,
    is the next layer's input on both sides.  Because codes and accumulators are exact and the
    float steps are the same single float32 operations, the chain stays identical to the end."""
    layers = I.config_resnet8_cifar(batch=4)
    lut = I.lut_random_error(2000)
    x0, _ = I.make_float_operands(layers[0], I.layer_seed(2, 0))
    xg = G.to_dev(x0)
    xo = x0
    ld = ax.lut_to_device(lut)
    for i, layer in enumerate(layers):
        _, w = I.make_float_operands(layer, I.layer_seed(2, i))
        relu = i > 0
        wd = G.to_dev(w)
        if i % 2:  # alternate between ranges handed in and ranges taken by the layer
            xr, wr = ax.ax_range_f32(xg, relu=relu), ax.ax_range_f32(wd)
        else:
            xr = wr = None
        acc, y = ax.ax_conv2d_f32(xg, wd, ld, layer.stride, layer.pad, xr, wr, relu=relu)
        torch.cuda.synchronize()
        ref = oracle.conv2d_f32(xo, w, lut, layer.stride, layer.pad, oracle.range_f32(xo, relu), oracle.range_f32(w),
                                relu=relu)
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref["acc"], ref["y"], "chained layer %d" % i)
        np.testing.assert_array_equal(y.cpu().numpy(), ref["y"])
        assert y.shape[1:] == (layers[i + 1].H, layers[i + 1].W, layers[i + 1].Cin) if i + 1 < len(layers) else True
        xg, xo = y, ref["y"]


def test_float_entry_points_reject_bad_arguments():
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    rng = torch.zeros(2, dtype=torch.float32, device="cuda")
    L_ = ax.lib()
    vp = lambda t: None if t is None else t.data_ptr()
    ws = torch.zeros(ax.ax_range_workspace_bytes(16), dtype=torch.uint8, device="cuda")
    assert L_.ax_range_f32(None, 16, 0, vp(rng), vp(ws), ws.numel(), None) == -1
    assert L_.ax_range_f32(vp(x), 0, 0, vp(rng), vp(ws), ws.numel(), None) == -2
    assert L_.ax_range_f32(vp(x), 16, 0, vp(rng), vp(ws), 8, None) == -5
    assert L_.ax_range_f32(vp(x), 16, 0, vp(rng), None, 0, None) == -5
    codes = torch.zeros(16, dtype=torch.uint8, device="cuda")
    assert L_.ax_quantize_f32(vp(x), 16, vp(rng), 0, 2, vp(codes), None, None) == -8
    assert L_.ax_quantize_f32(vp(x), 16, None, 0, 0, vp(codes), None, None) == -1
    assert L_.ax_quantize_f32(vp(x), 0, vp(rng), 0, 0, vp(codes), None, None) == -2
    with pytest.raises(ax.AxError):
        ax.ax_conv2d_f32(torch.zeros(1, 4, 4, 2, device="cuda"), torch.zeros(3, 3, 2, 2, device="cuda"),
                         ax.lut_to_device(I.lut_exact()), 1, 1, rng, rng, round_mode=5)
    with pytest.raises(ax.AxError):
        ax.ax_conv2d_f32(torch.zeros(1, 4, 4, 2, device="cuda"), torch.zeros(3, 3, 2, 2, device="cuda"),
                         ax.lut_to_device(I.lut_exact()), 1, 1, rng, rng,
                         workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()


EX_LAYERS = [
    # N, H, W, Cin, KH, KW, last, stride, pad, dilation, depthwise   (last = Cout, or the multiplier)
    (2, 9, 8, 5, 3, 3, 6, 1, 2, 2, False),
    (1, 40, 40, 16, 3, 3, 72, 1, 2, 2, False),              # table-tile path, implicit patch view
    (2, 30, 30, 20, 5, 5, 9, 2, 4, (2, 1), False),          # materialized patches
    (1, 7, 7, 256, 3, 3, 512, 1, 1, 1, False),              # lanes over channels when chosen
    (2, 8, 8, 6, 3, 3, 2, 1, 1, 1, True),
    (8, 56, 56, 64, 3, 3, 1, 1, 1, 1, True),                # depthwise kernel with the table in LDS
]


@pytest.mark.parametrize("variant", [0, 1, 3])
@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", EX_LAYERS, ids=lambda c: "x".join(str(v) for v in c[:7]) + ("_dw" if c[10] else ""))
def test_float_layer_with_the_full_parameter_set(case, signed, variant):
    N, H, W, Cin, KH, KW, last, s, p, d, dwise = case
    ax.ax_set_option("variant", variant)
    rng = np.random.default_rng(600 + Cin + last)
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    w = (rng.standard_normal((KH, KW, Cin, last)) * 0.2).astype(np.float32)
    relu = not signed
    lut = I.lut_signed_random_error(21) if signed else I.lut_random_error(21)
    given = variant == 1  # ranges handed in for one of the variants, taken by the layer otherwise
    xd, wd = G.to_dev(x), G.to_dev(w)
    xr = ax.ax_range_f32(xd, relu=relu) if given else None
    wr = ax.ax_range_f32(wd) if given else None
    acc, y = ax.ax_conv2d_f32_ex(xd, wd, ax.lut_to_device(lut), s, p, xr, wr, relu=relu, round_mode=int(signed),
                                 dilation=d, depthwise=dwise, signed=signed)
    torch.cuda.synchronize()
    ref = oracle.conv2d_f32_ex(x, w, lut, s, p, oracle.range_f32(x, relu), oracle.range_f32(w), relu=relu,
                               round_mode=int(signed), dilation=d, depthwise=dwise, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref["acc"], ref["y"], str(case))
    np.testing.assert_array_equal(y.cpu().numpy(), ref["y"])
