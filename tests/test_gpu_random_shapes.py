"""Seeded random geometries and option combinations through every convolution entry point,
against the oracle (int32 accumulators bit exact, floats within 1e-5 relative + 1e-6 absolute).
Shapes are small enough for the oracle and large enough to span several tiles now and then."""

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
    for name in ("variant", "split_k", "tile", "row_tiles", "share_order", "combine", "tables"):
        ax.ax_set_option(name, 0)


def _geometry(rng):
    kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    dh, dw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    sh, sw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    ph, pw = int(rng.integers(0, 5)), int(rng.integers(0, 5))
    H = int(rng.integers(dh * (kh - 1) + 1, dh * (kh - 1) + 24))
    W = int(rng.integers(dw * (kw - 1) + 1, dw * (kw - 1) + 24))
    cin = int(rng.choice([1, 3, 5, 16, 20, 32, 48, 64, 100]))
    cout = int(rng.choice([1, 4, 7, 8, 16, 24, 40, 64, 130]))
    n = int(rng.integers(1, 5))
    return n, H, W, cin, kh, kw, cout, (sh, sw), (ph, pw), (dh, dw)


@pytest.mark.parametrize("seed", range(48))
def test_random_layers_and_options(seed):
    rng = np.random.default_rng(7000 + seed)
    n, H, W, cin, kh, kw, cout, s, p, d = _geometry(rng)
    signed = bool(rng.integers(0, 2))
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    x = rng.integers(lo, hi, (n, H, W, cin)).astype(dt)
    x[rng.random(x.shape) < 0.4] = dt(lo + 3)
    w = rng.integers(lo, hi, (kh, kw, cin, cout)).astype(dt)
    q = I.Quant(0.013, int(rng.integers(lo, hi)), 0.0071, int(rng.integers(lo, hi)),
                None if rng.integers(0, 2) else int(rng.integers(lo, hi)))
    lut = I.lut_signed_random(seed) if signed else I.lut_random(seed)
    ax.ax_set_option("variant", int(rng.choice([0, 0, 2, 3, 1])))
    ax.ax_set_option("tile", int(rng.integers(0, 8)))
    ax.ax_set_option("split_k", int(rng.choice([0, 0, 2, 3, 5])))
    ax.ax_set_option("row_tiles", int(rng.choice([0, 0, 1, 2, 7])))
    ax.ax_set_option("share_order", seed % 3)  # not drawn from rng: the cases above stay what they were
    ax.ax_set_option("combine", (seed // 3) % 3)
    ax.ax_set_option("tables", (seed // 2) % 3)
    # now and then operands and outputs that are not 16-byte aligned
    off = int(rng.choice([0, 0, 1, 4]))
    xbuf = torch.zeros(x.size + 16, dtype=torch.int8 if signed else torch.uint8, device="cuda")
    xd = xbuf[off:off + x.size].view(x.shape)
    xd.copy_(G.to_dev(x))
    OH = (H + 2 * p[0] - d[0] * (kh - 1) - 1) // s[0] + 1
    OW = (W + 2 * p[1] - d[1] * (kw - 1) - 1) // s[1] + 1
    n_out = n * OH * OW * cout
    obuf_a = torch.zeros(n_out + 4, dtype=torch.int32, device="cuda")
    obuf_y = torch.zeros(n_out + 4, dtype=torch.float32, device="cuda")
    oo = int(rng.choice([0, 0, 1]))
    acc, y = ax.ax_conv2d_ex(xd, G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d,
                             acc_out=obuf_a[oo:oo + n_out], y_out=obuf_y[oo:oo + n_out])
    torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "seed %d" % seed)


@pytest.mark.parametrize("seed", range(16))
def test_random_layers_against_several_tables(seed):
    rng = np.random.default_rng(8000 + seed)
    n, H, W, cin, kh, kw, cout, s, p, d = _geometry(rng)
    OH = (H + 2 * p[0] - (kh - 1) - 1) // s[0] + 1
    OW = (W + 2 * p[1] - (kw - 1) - 1) // s[1] + 1
    if OH <= 0 or OW <= 0:
        pytest.skip("empty output for the undilated kernel")
    x = rng.integers(0, 256, (n, H, W, cin)).astype(np.uint8)
    w = rng.integers(0, 256, (kh, kw, cin, cout)).astype(np.uint8)
    q = I.Quant(0.02, int(rng.integers(0, 256)), 0.01, int(rng.integers(0, 256)), -1)
    T = int(rng.integers(1, 6))
    tabs = [np.ascontiguousarray(I.lut_random(100 * seed + t)).reshape(-1) for t in range(T)]
    ax.ax_set_option("variant", int(rng.choice([0, 2, 3])))
    ax.ax_set_option("tile", int(rng.integers(0, 8)))
    ax.ax_set_option("split_k", int(rng.choice([0, 0, 2, 3])))
    ax.ax_set_option("share_order", seed % 3)
    acc, y = ax.ax_conv2d_multi_lut(G.to_dev(x), G.to_dev(w), torch.stack([ax.lut_to_device(t) for t in tabs]), s, p, q)
    torch.cuda.synchronize()
    for t in range(T):
        acc_ref, y_ref = oracle.conv2d(x, w, tabs[t], s, p, q)
        G.assert_parity(acc[t].cpu().numpy(), y[t].cpu().numpy(), acc_ref, y_ref, "seed %d table %d" % (seed, t))


@pytest.mark.parametrize("seed", range(16))
def test_random_float_layers(seed):
    rng = np.random.default_rng(9000 + seed)
    n, H, W, cin, kh, kw, cout, s, p, d = _geometry(rng)
    signed = bool(rng.integers(0, 2))
    relu = bool(rng.integers(0, 2))
    mode = int(rng.integers(0, 2))
    x = (rng.standard_normal((n, H, W, cin)) * rng.uniform(0.1, 5.0) + rng.uniform(-1, 1)).astype(np.float32)
    w = (rng.standard_normal((kh, kw, cin, cout)) * 0.3).astype(np.float32)
    lut = I.lut_signed_random_error(seed) if signed else I.lut_random_error(seed)
    ax.ax_set_option("variant", int(rng.choice([0, 0, 2, 3, 1])))
    acc, y = ax.ax_conv2d_f32_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, relu=relu, round_mode=mode,
                                 dilation=d, signed=signed)
    torch.cuda.synchronize()
    ref = oracle.conv2d_f32_ex(x, w, lut, s, p, oracle.range_f32(x, relu), oracle.range_f32(w), relu=relu,
                               round_mode=mode, dilation=d, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref["acc"], ref["y"], "seed %d" % seed)
    np.testing.assert_array_equal(y.cpu().numpy(), ref["y"])


@pytest.mark.parametrize("seed", range(24))
def test_random_grouped_and_transposed_layers(seed):
    """Random geometries through the grouped form of ax_conv2d_ex and through ax_conv2d_transpose
    (with random tuning for the inner stride-1 layer of the latter)."""
    rng = np.random.default_rng(9000 + seed)
    signed = bool(rng.integers(0, 2))
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    lut = I.lut_signed_random(seed) if signed else I.lut_random(seed)
    q = I.Quant(0.013, int(rng.integers(lo, hi)), 0.0071, int(rng.integers(lo, hi)),
                None if rng.integers(0, 2) else int(rng.integers(lo, hi)))
    if seed % 2 == 0:
        n, H, W, _, kh, kw, _, s, p, d = _geometry(rng)
        groups = int(rng.choice([2, 3, 4, 8]))
        cin, cout = groups * int(rng.integers(1, 9)), groups * int(rng.integers(1, 7))
        x = rng.integers(lo, hi, (n, H, W, cin)).astype(dt)
        w = rng.integers(lo, hi, (kh, kw, cin // groups, cout)).astype(dt)
        acc, y = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d, groups=groups)
        torch.cuda.synchronize()
        acc_ref, y_ref = oracle.conv2d_grouped(x, w, lut, s, p, q, groups=groups, dilation=d, signed=signed)
    else:
        kh, kw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        d = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        s = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        p = (int(rng.integers(0, d[0] * (kh - 1) + 1)), int(rng.integers(0, d[1] * (kw - 1) + 1)))
        n, H, W = int(rng.integers(1, 4)), int(rng.integers(1, 12)), int(rng.integers(1, 12))
        cin = int(rng.choice([1, 3, 16, 20, 32, 64]))
        cout = int(rng.choice([1, 4, 8, 24, 40]))
        x = rng.integers(lo, hi, (n, H, W, cin)).astype(dt)
        w = rng.integers(lo, hi, (kh, kw, cin, cout)).astype(dt)
        if (H - 1) * s[0] + 1 + d[0] * (kh - 1) - 2 * p[0] <= 0 or (W - 1) * s[1] + 1 + d[1] * (kw - 1) - 2 * p[1] <= 0:
            pytest.skip("empty output")
        ax.ax_set_option("variant", int(rng.choice([0, 0, 2, 3, 1])))
        ax.ax_set_option("tile", int(rng.integers(0, 8)))
        ax.ax_set_option("split_k", int(rng.choice([0, 0, 2, 3])))
        acc, y = ax.ax_conv2d_transpose(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d)
        torch.cuda.synchronize()
        acc_ref, y_ref = oracle.conv2d_transpose(x, w, lut, s, p, q, dilation=d, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "seed %d" % seed)
