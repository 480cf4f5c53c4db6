"""GPU parity of ax_conv2d_multi_lut: one layer against several multiplier tables in one call.
Every table's result must be what the oracle (and the single-table call) gives for that table:
int32 accumulators bit exact, float outputs within 1e-5 relative + 1e-6 absolute."""

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


def L(N, H, W, Cin, KH, KW, Cout, s=1, p=0, x_dist="relu", w_dist="normal"):
    return I.Layer("m%dx%dx%dx%d_k%dx%d_c%d_s%d_p%d" % (N, H, W, Cin, KH, KW, Cout, s, p),
                   N, H, W, Cin, KH, KW, Cout, s, p, x_dist=x_dist, w_dist=w_dist)


def _tables(T, seed):
    kinds = [lambda s: I.lut_random_error(s), lambda s: I.lut_random(s), lambda s: I.lut_truncated(s % 9),
             lambda s: I.lut_exact(), lambda s: I.lut_const(s % 7)]
    return [np.ascontiguousarray(kinds[(seed + t) % len(kinds)](seed + t)).reshape(-1) for t in range(T)]


def _check(layer, T, seed, **kw):
    x, w, q = I.make_operands(layer, seed)
    tabs = _tables(T, seed)
    luts_d = torch.stack([ax.lut_to_device(t) for t in tabs])
    acc, y = ax.ax_conv2d_multi_lut(G.to_dev(x), G.to_dev(w), luts_d, layer.stride, layer.pad, q, **kw)
    torch.cuda.synchronize()
    acc, y = acc.cpu().numpy(), y.cpu().numpy()
    assert acc.shape[0] == T
    for t in range(T):
        acc_ref, y_ref = oracle.conv2d(x, w, tabs[t], layer.stride, layer.pad, q)
        G.assert_parity(acc[t], y[t], acc_ref, y_ref, "%s table %d of %d" % (layer.name, t, T))


LAYERS = [
    L(1, 5, 5, 1, 3, 3, 1, 1, 1),                 # one-thread-per-output kernel, table by table
    L(2, 9, 7, 5, 3, 3, 6, 2, 1),
    L(1, 40, 40, 16, 3, 3, 72, 1, 1),             # several ragged channel tiles
    L(2, 30, 30, 20, 5, 5, 9, 2, 2),              # materialized patches
    L(2, 14, 14, 256, 1, 1, 520, 1, 0),
    L(1, 7, 7, 512, 3, 3, 512, 1, 1),             # few pixels, many channels
    L(3, 28, 28, 64, 3, 3, 64, 1, 1),
]


@pytest.mark.parametrize("T", [1, 2, 5])
@pytest.mark.parametrize("variant", [0, 2, 3])
@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name)
def test_every_table_matches_the_oracle(layer, variant, T):
    ax.ax_set_option("variant", variant)
    _check(layer, T, 900 + layer.Cout + T)


def test_many_tables_fill_the_machine_with_whole_tiles():
    layer = L(2, 28, 28, 128, 3, 3, 128, 1, 1)
    _check(layer, 17, 77)


@pytest.mark.parametrize("opt", [("split_k", 2), ("split_k", 5), ("row_tiles", 3), ("tile", 3), ("tile", 2), ("tile", 6)])
def test_forced_decompositions_with_several_tables(opt):
    ax.ax_set_option(*opt)
    _check(L(1, 32, 32, 64, 3, 3, 40, 1, 1), 3, 55)
    ax.ax_set_option("variant", 3)
    _check(L(1, 6, 6, 64, 1, 1, 300, 1, 0), 4, 56)


def test_result_is_the_single_table_call_bit_for_bit_and_optional_outputs():
    layer = L(2, 20, 20, 32, 3, 3, 48, 1, 1)
    x, w, q = I.make_operands(layer, 5)
    tabs = _tables(4, 5)
    xd, wd = G.to_dev(x), G.to_dev(w)
    luts_d = torch.stack([ax.lut_to_device(t) for t in tabs])
    acc, y = ax.ax_conv2d_multi_lut(xd, wd, luts_d, 1, 1, q)
    acc_only, none = ax.ax_conv2d_multi_lut(xd, wd, luts_d, 1, 1, q, y_out=False)
    assert none is None and torch.equal(acc_only, acc)
    for t in range(4):
        a1, y1 = ax.ax_conv2d(xd, wd, luts_d[t], 1, 1, q)
        assert torch.equal(a1, acc[t]) and torch.equal(y1, y[t])


def test_lut_sweep_layer_at_full_size_sampled():
    """The 3x3 layer of the table-sweep workload at batch 64 against 8 tables in one call."""
    layer = I.config_lut_sweep(batch=64)[1]
    x, w, q = I.make_operands(layer, I.layer_seed(4, 1))
    tabs = [np.ascontiguousarray(I.lut_random_error(sd)).reshape(-1) for sd in range(8)]
    luts_d = torch.stack([ax.lut_to_device(t) for t in tabs])
    acc, y = ax.ax_conv2d_multi_lut(G.to_dev(x), G.to_dev(w), luts_d, layer.stride, layer.pad, q)
    torch.cuda.synchronize()
    rng = np.random.default_rng(44)
    n_out = layer.M * layer.Cout
    for t in range(8):
        idx = np.concatenate([rng.integers(0, n_out, size=200), np.array([0, n_out - 1])]).astype(np.int64)
        a_ref, y_ref = oracle.conv2d_sample(x, w, tabs[t], layer.stride, layer.pad, q, idx)
        ti = torch.from_numpy(idx).cuda()
        G.assert_parity(acc[t].reshape(-1)[ti].cpu().numpy(), y[t].reshape(-1)[ti].cpu().numpy(), a_ref, y_ref,
                        "table %d" % t)


def test_bad_table_counts_are_rejected():
    L_ = ax.lib()
    assert L_.ax_conv2d_multi_lut_workspace_bytes(1, 8, 8, 16, 3, 3, 16, 0, 1, 1, 1, 1) == 0
    assert L_.ax_conv2d_multi_lut_workspace_bytes(1, 8, 8, 16, 3, 3, 16, 70000, 1, 1, 1, 1) == 0
    x = torch.zeros((1, 8, 8, 16), dtype=torch.uint8, device="cuda")
    w = torch.zeros((3, 3, 16, 16), dtype=torch.uint8, device="cuda")
    luts = torch.zeros((0, 65536), dtype=torch.int16, device="cuda")
    with pytest.raises(ax.AxError):
        ax.ax_conv2d_multi_lut(x, w, luts, 1, 1, I.Quant(), workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
