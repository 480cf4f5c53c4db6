"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded operands.  int32 accumulators bit exact; float outputs within
1e-5 relative + 1e-6 absolute."""

import numpy as np
import pytest
import torch

from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu

VARIANTS = [0, 1, 2, 3]


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    ax.ax_set_option("variant", 0)
    ax.ax_set_option("split_k", 0)
    ax.ax_set_option("tile", 0)
    ax.ax_set_option("row_tiles", 0)
    ax.ax_set_option("share_order", 0)
    ax.ax_set_option("combine", 0)
    ax.ax_set_option("tables", 0)


def L(N, H, W, Cin, KH, KW, Cout, s=1, p=0, dense=False, x_dist="uniform", w_dist="uniform", name=None):
    return I.Layer(name or "t%dx%dx%dx%d_k%dx%d_c%d_s%d_p%d" % (N, H, W, Cin, KH, KW, Cout, s, p),
                   N, H, W, Cin, KH, KW, Cout, s, p, dense=dense, x_dist=x_dist, w_dist=w_dist)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("table", ["truncated4", "exact"])
def test_config1_single_layer(variant, table):
    ax.ax_set_option("variant", variant)
    lut = I.lut_truncated(4) if table == "truncated4" else I.lut_exact()
    G.check_layer(I.config_single_layer()[0], I.layer_seed(1, 0), lut)


@pytest.mark.parametrize("variant", VARIANTS)
def test_config2_cifar_stack_small_batch(variant):
    ax.ax_set_option("variant", variant)
    lut = I.lut_random_error(2000)
    for i, layer in enumerate(I.config_resnet8_cifar(batch=5)):
        G.check_layer(layer, I.layer_seed(2, i), lut)


EDGE = [
    L(1, 1, 1, 1, 1, 1, 1),                       # a single multiply
    L(1, 5, 5, 1, 3, 3, 1, 1, 1),
    L(2, 9, 7, 5, 3, 3, 6, 2, 1),                 # odd channel counts, stride 2
    L(1, 4, 4, 2, 3, 3, 2, 1, 3),                 # padding wider than the kernel
    L(2, 7, 5, 3, 2, 3, 5, 3, 2),                 # non-square kernel, stride 3
    L(3, 11, 13, 16, 3, 3, 10, 1, 1),             # Cout not a multiple of 8
    L(1, 40, 40, 16, 3, 3, 72, 1, 1),             # more than one channel tile, ragged
    L(1, 33, 35, 32, 1, 1, 24, 1, 0),             # ragged pixel tile
    L(2, 30, 30, 20, 5, 5, 9, 2, 2),              # Cin not a multiple of 16
    L(1, 64, 64, 3, 7, 7, 16, 2, 3),              # stem-like: Cin = 3
    L(1, 12, 12, 64, 3, 3, 130, 1, 1),
    L(1, 2, 2, 512, 2, 2, 256, 1, 0),             # one output pixel per image, long K
    L(70, 1, 1, 96, 1, 1, 40, dense=True),        # dense, ragged everywhere
    L(1, 1, 1, 64, 1, 1, 1000, dense=True),       # a single row
    L(1300, 1, 1, 17, 1, 1, 3, dense=True),
]


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("layer", EDGE, ids=lambda l: l.name)
def test_edge_shapes(variant, layer):
    ax.ax_set_option("variant", variant)
    G.check_layer(layer, 77, I.lut_random(9))


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("split_k", [2, 3, 7])
def test_forced_k_slices(variant, split_k):
    """Output tiles shared by several workgroups (combined by the fix-up kernel)."""
    ax.ax_set_option("variant", variant)
    ax.ax_set_option("split_k", split_k)
    G.check_layer(L(1, 14, 14, 64, 3, 3, 72, 1, 1, x_dist="relu", w_dist="normal"), 5, I.lut_random_error(3))
    G.check_layer(L(40, 1, 1, 1000, 1, 1, 130, dense=True), 6, I.lut_truncated(6))


@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("rows", [1, 2, 3, 5, 40, 100000])
def test_forced_row_tile_counts(variant, rows):
    """The lane dimension cut into more (lower) tiles than it needs, incl. counts that leave the
    last tile nearly empty and counts beyond what the layer allows (clamped)."""
    ax.ax_set_option("variant", variant)
    ax.ax_set_option("row_tiles", rows)
    lut = I.lut_random(23)
    G.check_layer(L(2, 50, 47, 32, 3, 3, 72, 1, 1), 41, lut)           # 4700 pixels: 3 tiles at least
    G.check_layer(L(1, 20, 20, 48, 1, 1, 30, 2, 0), 42, lut)
    ax.ax_set_option("split_k", 2)
    G.check_layer(L(1, 64, 64, 64, 3, 3, 40, 1, 1), 43, lut)


@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("split_k", [0, 1, 3, 8])
def test_share_numberings(variant, order, split_k):
    """Workgroups take their shares of the (tile, chunk) space in launch order or XCD by XCD;
    grids that are and are not multiples of eight, with and without shared tiles."""
    ax.ax_set_option("variant", variant)
    ax.ax_set_option("share_order", order)
    ax.ax_set_option("split_k", split_k)
    lut = I.lut_random(29)
    G.check_layer(L(3, 40, 41, 32, 3, 3, 72, 1, 1), 51, lut)           # 4920 pixels x 72 channels
    G.check_layer(L(1, 20, 20, 48, 1, 1, 30, 2, 0), 52, lut)           # a single tile
    G.check_layer(L(37, 1, 1, 600, 1, 1, 333, dense=True), 53, lut)
    G.check_layer(L(2, 33, 33, 16, 5, 5, 24, 2, 2, x_dist="relu", w_dist="normal"), 54, I.lut_truncated(6))


@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("combine", [1, 2])
@pytest.mark.parametrize("split_k", [0, 2, 3, 7, 16])
def test_shared_tiles_combined_by_either_kernel(variant, combine, split_k):
    """Tiles whose sum over the taps is shared by several workgroups: pieces added by the second
    kernel or by the workgroup that finishes a tile last, from two to sixteen pieces per tile;
    twice in a row, since the arrival counters must be back at zero after a call."""
    ax.ax_set_option("variant", variant)
    ax.ax_set_option("combine", combine)
    ax.ax_set_option("split_k", split_k)
    lut = I.lut_random(33)
    for rep in range(2):
        G.check_layer(L(3, 40, 41, 32, 3, 3, 72, 1, 1), 61 + rep, lut)
        G.check_layer(L(1, 7, 7, 512, 3, 3, 512, 1, 1), 63 + rep, lut)      # few pixels: K slices by default
        G.check_layer(L(37, 1, 1, 600, 1, 1, 333, dense=True), 65 + rep, lut)
        G.check_layer(L(2, 33, 33, 16, 5, 5, 24, 2, 2, x_dist="relu", w_dist="normal"), 67 + rep, I.lut_truncated(6))


@pytest.mark.parametrize("tables", [1, 2])
@pytest.mark.parametrize("tile", [3, 5])
@pytest.mark.parametrize("split_k", [0, 3])
def test_tables_assembled_in_the_kernel_or_ready_made(tables, tile, split_k):
    """The per-tap tables of the table-tile kernel: built in LDS from the rows of the multiplier
    table, or copied ready-made from the prepared block; ragged K (taps past the end of the sum),
    ragged channel tiles, materialized patches, K slices."""
    ax.ax_set_option("variant", 2)
    ax.ax_set_option("tables", tables)
    ax.ax_set_option("tile", tile)
    ax.ax_set_option("split_k", split_k)
    lut = I.lut_random(35)
    G.check_layer(L(3, 40, 41, 32, 3, 3, 72, 1, 1), 71, lut)
    G.check_layer(L(2, 30, 30, 20, 5, 5, 9, 2, 2), 72, lut)             # Cin % 16 != 0: K padded to 512
    G.check_layer(L(1, 7, 7, 512, 3, 3, 130, 1, 1), 73, I.lut_truncated(6))
    G.check_layer(L(40, 1, 1, 100, 1, 1, 64, dense=True), 74, lut)
    G.check_layer(L(128, 32, 32, 16, 3, 3, 16, 1, 1, x_dist="relu", w_dist="normal"), 75, I.lut_random_error(7))


TILES = list(range(1, 8))


@pytest.mark.parametrize("variant", [2, 3])
@pytest.mark.parametrize("tile", TILES)
def test_tile_configurations(variant, tile):
    """Every table-tile configuration (threads, lane elements, groups, taps per barrier)."""
    ax.ax_set_option("variant", variant)
    ax.ax_set_option("tile", tile)
    lut = I.lut_random(21)
    G.check_layer(L(2, 30, 33, 32, 3, 3, 72, 1, 1), 31, lut)           # ragged pixel and channel tiles
    G.check_layer(L(1, 20, 20, 48, 1, 1, 30, 2, 0), 32, lut)           # Cout not a multiple of 4: scalar stores
    G.check_layer(L(3, 9, 9, 7, 3, 3, 16, 1, 1), 33, lut)              # materialized patches, K tail
    ax.ax_set_option("split_k", 3)
    G.check_layer(L(1, 16, 16, 64, 3, 3, 40, 1, 1), 34, lut)
    G.check_layer(L(50, 1, 1, 200, 1, 1, 64, dense=True), 35, lut)


RESNET_SLICES = [
    L(1, 224, 224, 3, 7, 7, 64, 2, 3, name="conv1"),
    L(2, 56, 56, 64, 1, 1, 64, x_dist="relu", w_dist="normal", name="s1.a1x1"),
    L(1, 56, 56, 64, 3, 3, 64, 1, 1, x_dist="relu", w_dist="normal", name="s1.b3x3"),
    L(1, 56, 56, 128, 3, 3, 128, 2, 1, x_dist="relu", w_dist="normal", name="s2.b3x3s2"),
    L(1, 56, 56, 256, 1, 1, 512, 2, 0, x_dist="relu", w_dist="normal", name="s2.proj"),
    L(2, 14, 14, 1024, 1, 1, 256, x_dist="relu", w_dist="normal", name="s3.a1x1"),
    L(2, 7, 7, 512, 3, 3, 512, 1, 1, x_dist="relu", w_dist="normal", name="s4.b3x3"),
    L(2, 7, 7, 512, 1, 1, 2048, x_dist="relu", w_dist="normal", name="s4.c1x1"),
    L(32, 1, 1, 2048, 1, 1, 1000, dense=True, x_dist="relu", w_dist="normal", name="fc"),
]


@pytest.mark.parametrize("variant", [0, 2, 3])
@pytest.mark.parametrize("layer", RESNET_SLICES, ids=lambda l: l.name)
def test_config3_resnet50_shapes_small_batch(variant, layer):
    ax.ax_set_option("variant", variant)
    G.check_layer(layer, 3000, I.lut_truncated(6))


@pytest.mark.parametrize("variant", [0, 2, 3])
def test_config4_layers_two_tables(variant):
    ax.ax_set_option("variant", variant)
    for i, layer in enumerate(I.config_lut_sweep(batch=1)):
        for lut_seed in (0, 63):
            G.check_layer(layer, I.layer_seed(4, i), I.lut_random_error(lut_seed))


@pytest.mark.parametrize("variant", [0, 2, 3])
def test_config5_gemm_shaped_small(variant):
    ax.ax_set_option("variant", variant)
    conv = L(1, 14, 14, 1024, 1, 1, 2048, name="c5.conv1x1")
    fc = L(24, 1, 1, 4096, 1, 1, 4096, dense=True, name="c5.fc")
    for lut in (I.lut_exact(), I.lut_truncated(6)):
        G.check_layer(conv, I.layer_seed(5, 0), lut)
        G.check_layer(fc, I.layer_seed(5, 1), lut)


@pytest.mark.parametrize("variant", VARIANTS)
def test_special_tables_on_gpu(variant):
    """Zero table, one-hot table (counts padded taps), non-commutative tables."""
    ax.ax_set_option("variant", variant)
    layer = L(2, 10, 9, 16, 3, 3, 24, 1, 1)
    q = I.Quant(0.5, 200, 0.25, 3, 200)
    x, w, _ = I.make_operands(layer, 8)
    x[x == 200] = 199
    w[:, :, 0, ::3] = 99
    for lut in (I.lut_zero(), I.lut_onehot(200, 99), I.lut_first_operand(), I.lut_second_operand(), I.lut_const(65535)):
        acc, y = G.run_gpu(x, w, lut, 1, 1, q)
        acc_ref, y_ref = G.run_oracle(x, w, lut, 1, 1, q)
        G.assert_parity(acc, y, acc_ref, y_ref)
    acc, _ = G.run_gpu(x, w, I.lut_onehot(200, 99), 1, 1, q)
    assert acc[0, 0, 0, 0] > 0 and acc[0, 5, 4, 0] == 0  # only border pixels see the pad code


@pytest.mark.parametrize("variant", VARIANTS)
def test_accumulator_near_int32_limit(variant):
    """K = 32768 with every entry 65535: acc = 2147450880, just below 2^31."""
    ax.ax_set_option("variant", variant)
    layer = L(3, 1, 1, 32768, 1, 1, 9, dense=True)
    x, w, q = I.make_operands(layer, 1)
    acc, y = G.run_gpu(x, w, I.lut_const(65535), 1, 0, q, dense=True)
    assert np.all(acc == 2147450880)
    acc_ref, y_ref = G.run_oracle(x, w, I.lut_const(65535), 1, 0, q, dense=True)
    G.assert_parity(acc, y, acc_ref, y_ref)


@pytest.mark.parametrize("variant", [0, 1, 2])
def test_optional_outputs_and_errors(variant):
    ax.ax_set_option("variant", variant)
    layer = L(1, 20, 20, 16, 3, 3, 16, 1, 1)
    x, w, q = I.make_operands(layer, 2)
    lut = I.lut_random_error(1)
    acc_ref, y_ref = G.run_oracle(x, w, lut, 1, 1, q)
    acc, y = G.run_gpu(x, w, lut, 1, 1, q, y_out=False)
    assert y is None and np.array_equal(acc, acc_ref)
    acc, y = G.run_gpu(x, w, lut, 1, 1, q, acc_out=False)
    assert acc is None
    G.assert_parity(acc_ref, y, acc_ref, y_ref)
    with pytest.raises(ax.AxError) as e:
        G.run_gpu(x, w, lut, 1, 1, q, acc_out=False, y_out=False)
    assert e.value.code == -1
    big = L(2, 56, 56, 64, 3, 3, 64, 1, 1)
    xb, wb, qb = I.make_operands(big, 3)
    if ax.ax_get_option("variant") != 1 and ax.ax_conv2d_workspace_bytes(xb.shape, wb.shape, 1, 1) > 256:
        with pytest.raises(ax.AxError) as e:
            G.run_gpu(xb, wb, lut, 1, 1, qb, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
        assert e.value.code == -5


def test_repeatable_and_stream():
    """Two runs give identical bits (integer sums are order independent, so any difference
    would be a race), also on a non-default stream with a reused workspace."""
    layer = L(2, 28, 28, 128, 3, 3, 128, 1, 1, x_dist="relu", w_dist="normal")
    x, w, q = I.make_operands(layer, 4)
    lut = I.lut_random_error(2)
    xd, wd, ld = G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut)
    ws = torch.empty(ax.ax_conv2d_workspace_bytes(x.shape, w.shape, 1, 1), dtype=torch.uint8, device="cuda")
    a1, y1 = ax.ax_conv2d(xd, wd, ld, 1, 1, q, workspace=ws)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        a2, y2 = ax.ax_conv2d(xd, wd, ld, 1, 1, q, workspace=ws)
    s.synchronize()
    assert torch.equal(a1, a2) and torch.equal(y1, y2)
    acc_ref, y_ref = G.run_oracle(x, w, lut, 1, 1, q)
    G.assert_parity(a2.cpu().numpy(), y2.cpu().numpy(), acc_ref, y_ref)
