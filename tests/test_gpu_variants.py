"""GPU parity of the operator variants (dilation, signed codes and tables, depthwise) through
ax_conv2d_ex against the CPU oracle: int32 accumulators bit exact, float outputs within
1e-5 relative + 1e-6 absolute."""

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


def _operands(shape, seed, signed, depthwise=False, mult=1):
    N, H, W, Cin, KH, KW, Cout = shape
    rng = np.random.default_rng(seed)
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    x = rng.integers(lo, hi, (N, H, W, Cin)).astype(dt)
    # half of the activations at one value, like post-ReLU tensors
    x[rng.random(x.shape) < 0.5] = dt(lo + 5)
    wshape = (KH, KW, Cin, mult) if depthwise else (KH, KW, Cin, Cout)
    w = rng.integers(lo, hi, wshape).astype(dt)
    q = I.Quant(0.021, int(rng.integers(lo, hi)), 0.0043, int(rng.integers(lo, hi)),
                None if seed % 2 else int(rng.integers(lo, hi)))
    return x, w, q


def _check(x, w, lut, s, p, d, q, depthwise=False, what=""):
    signed = x.dtype == np.int8
    acc, y = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), s, p, q, dilation=d, depthwise=depthwise)
    torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_ex(x, w, lut, s, p, q, dilation=d, depthwise=depthwise, signed=signed)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, what)


SHAPES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad, dilation
    ((1, 1, 1, 1, 1, 1, 1), 1, 0, 1),
    ((2, 9, 7, 5, 3, 3, 6), 2, 1, 1),
    ((1, 12, 12, 4, 3, 3, 5), 1, 2, 2),
    ((2, 11, 9, 3, 3, 2, 4), 2, 3, 3),
    ((2, 20, 20, 16, 3, 3, 24), 1, (2, 4), (2, 4)),        # implicit patch reads, dilation differs per axis
    ((1, 40, 40, 32, 3, 3, 72), 1, 2, 2),                  # several channel tiles
    ((2, 30, 30, 20, 5, 5, 9), 2, 4, 2),                   # materialized patches (Cin % 16 != 0)
    ((1, 7, 7, 256, 3, 3, 512), 1, 3, 3),                  # few pixels, many channels
    ((4, 14, 14, 64, 1, 1, 200), 1, 0, 1),
]


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", SHAPES, ids=lambda c: "x".join(map(str, c[0])) + "_d%s" % (c[3],))
def test_dilated_and_signed_layers(case, signed, variant):
    shape, s, p, d = case
    ax.ax_set_option("variant", variant)
    x, w, q = _operands(shape, 100 + shape[3] + variant, signed)
    lut = I.lut_signed_random_error(5) if signed else I.lut_random_error(5)
    _check(x, w, lut, s, p, d, q, what=str(case))


MATERIALIZED = [
    # patches copied out by the staged kernel (input rows in LDS) ...
    ((3, 37, 70, 3, 7, 7, 16), 2, 3, 1),                   # stem-like, three stripes per row, the last ragged
    ((2, 19, 33, 5, 3, 5, 8), (1, 2), (2, 0), (2, 3)),     # dilation, stride and padding differ per axis
    ((1, 9, 150, 1, 1, 3, 8), 1, (0, 40), 1),              # stripes that read padding columns only
    ((2, 16, 16, 24, 3, 3, 16), 1, 1, 1),                  # Cin % 16 == 8
    ((1, 12, 12, 100, 7, 7, 8), 1, 3, 1),                  # ... and by the one-thread-per-piece kernel: long patch
    ((1, 10, 10, 20, 3, 3, 8), 1, 40, 36),                 # widely dilated, still staged
    ((1, 10, 10, 20, 3, 3, 8), 1, 150, 150),               # dilated beyond what the stage holds
]


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", MATERIALIZED, ids=lambda c: "x".join(map(str, c[0])) + "_d%s" % (c[3],))
def test_materialized_patches(case, signed):
    """Cin not a multiple of 16: the lane-side operand is written out by one of two kernels."""
    shape, s, p, d = case
    ax.ax_set_option("variant", 2)
    x, w, q = _operands(shape, 300 + shape[3], signed)
    lut = I.lut_signed_random(9) if signed else I.lut_random(9)
    _check(x, w, lut, s, p, d, q, what=str(case))


@pytest.mark.parametrize("table", ["exact", "random", "minimum"])
@pytest.mark.parametrize("variant", [1, 2, 3])
def test_signed_tables_of_either_sign(table, variant):
    """Arbitrary int16 entries (sums of either sign), and the table of all -32768: the most
    negative accumulator, -32768 * K."""
    ax.ax_set_option("variant", variant)
    shape = (2, 10, 10, 32, 3, 3, 40)
    x, w, q = _operands(shape, 7, True)
    lut = {"exact": I.lut_signed_exact(), "random": I.lut_signed_random(11),
           "minimum": np.full((256, 256), -32768, np.int16)}[table]
    _check(x, w, lut, 1, 1, 1, q, what=table)
    if table == "minimum":
        acc, _ = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), 1, 1, q)
        assert bool((acc == -32768 * 288).all())


@pytest.mark.parametrize("split", [2, 3])
@pytest.mark.parametrize("signed", [False, True])
def test_variants_with_forced_k_split(split, signed):
    ax.ax_set_option("split_k", split)
    shape = (1, 20, 20, 64, 3, 3, 64)
    x, w, q = _operands(shape, 31, signed)
    lut = I.lut_signed_random(3) if signed else I.lut_random(3)
    _check(x, w, lut, 1, 2, 2, q, what="split %d" % split)


def test_signed_long_k_wide_epilogue():
    """K above 16384 takes the 64-bit correction path."""
    shape = (1, 3, 3, 2048, 3, 3, 24)
    x, w, q = _operands(shape, 5, True)
    for variant in (2, 3):
        ax.ax_set_option("variant", variant)
        _check(x, w, I.lut_signed_random(9), 1, 1, 1, q, what="K=18432 variant %d" % variant)


DEPTHWISE = [
    # N, H, W, Cin, KH, KW, mult, stride, pad, dilation
    (1, 1, 1, 2, 1, 1, 2, 1, 0, 1),
    (2, 8, 7, 4, 3, 3, 1, 2, 1, 1),
    (2, 8, 7, 4, 3, 3, 3, 1, 1, 2),
    (4, 28, 28, 96, 3, 3, 1, 1, 1, 1),        # a MobileNet-like depthwise layer
    (2, 14, 14, 33, 5, 5, 2, 2, 2, 1),
]


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", DEPTHWISE, ids=lambda c: "x".join(map(str, c)))
def test_depthwise_layers(case, signed):
    N, H, W, Cin, KH, KW, mult, s, p, d = case
    x, w, q = _operands((N, H, W, Cin, KH, KW, Cin * mult), 200 + Cin, signed, depthwise=True, mult=mult)
    lut = I.lut_signed_random(13) if signed else I.lut_random(13)
    _check(x, w, lut, s, p, d, q, depthwise=True, what=str(case))


DEPTHWISE_LDS = [
    # large enough for the kernel that keeps the whole table in LDS
    (8, 56, 56, 64, 3, 3, 1, 1, 1, 1),
    (4, 57, 55, 36, 3, 3, 1, 2, 1, 1),        # ragged everything, stride 2
    (2, 64, 64, 32, 5, 5, 1, 1, 4, 2),        # 5x5, dilation 2
    (16, 28, 28, 128, 3, 3, 1, 1, 0, 1),      # no padding
    (8, 40, 40, 33, 3, 3, 2, 1, 1, 1),        # channel multiplier 2, 66 output channels: last group of a pixel is ragged
    (16, 48, 48, 6, 5, 5, 1, 1, 2, 1),        # channel count no multiple of four
    (16, 56, 56, 24, 3, 3, 4, 2, 1, 1),       # channel multiplier 4: a group of outputs reads one input channel
    (4, 30, 30, 50, 4, 2, 3, 1, 1, 2),        # 4x2 kernel, multiplier 3, dilation 2
]


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("case", DEPTHWISE_LDS, ids=lambda c: "x".join(map(str, c)))
def test_depthwise_layers_table_in_lds(case, signed, variant):
    """variant 0 takes the LDS-table depthwise kernel for these sizes, variant 1 forces the
    one-thread-per-output kernel; both must match the oracle."""
    ax.ax_set_option("variant", variant)
    N, H, W, Cin, KH, KW, mult, s, p, d = case
    x, w, q = _operands((N, H, W, Cin, KH, KW, Cin * mult), 300 + Cin, signed, depthwise=True, mult=mult)
    lut = I.lut_signed_random(17) if signed else I.lut_random(17)
    _check(x, w, lut, s, p, d, q, depthwise=True, what=str(case))


def test_depthwise_outputs_not_16_byte_aligned():
    N, H, W, Cin = 8, 56, 56, 64
    x, w, q = _operands((N, H, W, Cin, 3, 3, Cin), 9, False, depthwise=True)
    lut = I.lut_random(19)
    n_out = N * H * W * Cin
    acc_buf = torch.zeros(n_out + 1, dtype=torch.int32, device="cuda")
    y_buf = torch.zeros(n_out + 1, dtype=torch.float32, device="cuda")
    acc, y = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), 1, 1, q, depthwise=True,
                             acc_out=acc_buf[1:], y_out=y_buf[1:])
    torch.cuda.synchronize()
    acc_ref, y_ref = oracle.conv2d_ex(x, w, lut, 1, 1, q, depthwise=True)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "unaligned outputs")


def test_descriptor_with_defaults_is_the_plain_layer():
    layer = I.Layer("plain", 2, 16, 16, 32, 3, 3, 48, 1, 1, x_dist="relu", w_dist="normal")
    x, w, q = I.make_operands(layer, 3)
    lut = I.lut_truncated(5)
    a0, y0 = ax.ax_conv2d(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), 1, 1, q)
    a1, y1 = ax.ax_conv2d_ex(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), 1, 1, q)
    assert torch.equal(a0, a1) and torch.equal(y0, y1)


def test_descriptor_errors():
    L_ = ax.lib()
    x = torch.zeros((1, 4, 4, 2), dtype=torch.uint8, device="cuda")
    w = torch.zeros((3, 3, 2, 2), dtype=torch.uint8, device="cuda")
    lut = ax.lut_to_device(I.lut_exact())
    with pytest.raises(ax.AxError):  # dilated kernel larger than the padded image
        ax.ax_conv2d_ex(x, w, lut, 1, 0, I.Quant(), dilation=2)
    with pytest.raises(ax.AxError):  # signed zero point out of range
        ax.ax_conv2d_ex(x.to(torch.int8), w.to(torch.int8), lut, 1, 1, I.Quant(1.0, 200, 1.0, 0, None))
    # for signed layers -1 is a code, not "default": accepted
    ax.ax_conv2d_ex(x.to(torch.int8), w.to(torch.int8), lut, 1, 1, I.Quant(1.0, 0, 1.0, 0, -1))
    d = ax.ax_conv_desc_t(1, 4, 4, 2, 3, 3, 3, 1, 1, 1, 1, 1, 1, 1, 0)  # depthwise with Cout % Cin != 0
    assert L_.ax_conv2d_ex_workspace_bytes(d, None) == 0
    d = ax.ax_conv_desc_t(1, 4, 4, 2, 3, 3, 2, 1, 1, 1, 1, 1, 1, 2, 0)  # flag that is neither 0 nor 1
    assert L_.ax_conv2d_ex_workspace_bytes(d, None) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("M", [1, 16, 17, 32, 33, 64])
def test_dense_layers_of_few_rows(M, signed):
    """Dense layers of at most 64 rows take the kernel with the whole table in LDS (four output
    columns per workgroup, taps over the lanes): every rows-per-wave form, K that is and is not a
    multiple of 64, filters that are and are not dword aligned; as a 1 x 1 convolution, through
    the descriptor entry point and through a handle."""
    rng = np.random.default_rng(500 + M)
    lo, hi, dt = (-128, 128, np.int8) if signed else (0, 256, np.uint8)
    lut = I.lut_signed_random(M) if signed else I.lut_random_error(M)
    for K, Cout, off in ((2048, 1000, 0), (100, 256, 0), (640, 260, 1)):
        x = rng.integers(lo, hi, (M, 1, 1, K)).astype(dt)
        x[rng.random(x.shape) < 0.5] = dt(lo + 7)
        w = rng.integers(lo, hi, (1, 1, K, Cout)).astype(dt)
        q = I.Quant(0.017, int(rng.integers(lo, hi)), 0.0031, int(rng.integers(lo, hi)), None)
        wbuf = torch.zeros(w.size + 8, dtype=torch.int8 if signed else torch.uint8, device="cuda")
        wd = wbuf[off:off + w.size].view(w.shape)
        wd.copy_(G.to_dev(w))
        acc, y = ax.ax_conv2d_ex(G.to_dev(x), wd, ax.lut_to_device(lut), 1, 0, q)
        torch.cuda.synchronize()
        acc_ref, y_ref = oracle.conv2d_ex(x, w, lut, 1, 0, q, signed=signed)
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, "M %d K %d Cout %d" % (M, K, Cout))
        desc = ax._conv_desc(x.shape, w.shape, 1, 0, 1, False, signed)
        with ax.AxLayer(desc, q) as h:
            assert h.plan()["variant"] == 1  # not a table-tile layer
            h.prepare(wd, ax.lut_to_device(lut))
            acc2, y2 = h.run(G.to_dev(x))
            torch.cuda.synchronize()
            assert torch.equal(acc2, acc) and torch.equal(y2, y)
