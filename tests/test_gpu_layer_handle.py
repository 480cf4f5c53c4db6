"""GPU parity of the layer handles (ax_layer_*): filters and table prepared once, then several
calls with different activations.  Every call must give what the oracle gives for its
activations (int32 accumulators bit exact, float outputs within 1e-5 relative + 1e-6 absolute),
whatever kernel family, lane assignment or work decomposition the handle was created with."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu


def _tune(**kw):
    t = dict(variant=0, split_k=0, tile=0, row_tiles=0, share_order=0)
    t.update(kw)
    return t


def L(N, H, W, Cin, KH, KW, Cout, s=1, p=0, x_dist="relu", w_dist="normal"):
    return I.Layer("h%dx%dx%dx%d_k%dx%d_c%d_s%d_p%d" % (N, H, W, Cin, KH, KW, Cout, s, p),
                   N, H, W, Cin, KH, KW, Cout, s, p, x_dist=x_dist, w_dist=w_dist)


LAYERS = [
    L(1, 5, 5, 3, 3, 3, 4, 1, 1),                 # tiny: direct kernel, no prepared block
    L(2, 30, 30, 20, 5, 5, 9, 2, 2),              # materialized patches (Cin % 16 != 0): per-call preparation
    L(1, 40, 40, 16, 3, 3, 72, 1, 1),             # implicit patch view, ragged channel tiles
    L(2, 14, 14, 256, 1, 1, 520, 1, 0),
    L(1, 7, 7, 512, 3, 3, 512, 1, 1),             # few pixels, many channels: K slices and the fix-up pass
    L(3, 28, 28, 64, 3, 3, 64, 1, 1),
]
TUNES = [_tune(), _tune(variant=2, split_k=3), _tune(variant=3), _tune(variant=3, split_k=2, share_order=1),
         _tune(variant=2, tile=3, row_tiles=2), _tune(variant=1), _tune(variant=2, split_k=5, combine=1),
         _tune(variant=2, split_k=5, combine=2), _tune(variant=3, split_k=9, combine=2),
         _tune(variant=2, tables=2), _tune(variant=2, tile=3, tables=2, split_k=2), _tune(variant=2, tables=1)]


@pytest.mark.parametrize("li", range(len(LAYERS)))
@pytest.mark.parametrize("ti", range(len(TUNES)))
def test_prepared_layer_matches_oracle_on_every_call(li, ti):
    layer, tune = LAYERS[li], TUNES[ti]
    lut = I.lut_random_error(40 + li)
    x0, w, q = I.make_operands(layer, 7000 + li)
    wd, lut_d = G.to_dev(w), ax.lut_to_device(lut)
    desc = ax._conv_desc(x0.shape, w.shape, layer.stride, layer.pad)
    with ax.AxLayer(desc, q, tune=tune) as h:
        plan = h.plan()
        if tune["variant"]:
            assert plan["variant"] == tune["variant"]
        h.prepare(wd, lut_d)
        for call in range(3):
            x = x0 if call == 0 else I.make_operands(layer, 7100 + 10 * li + call)[0]
            acc, y = h.run(G.to_dev(x))
            torch.cuda.synchronize()
            acc_ref, y_ref = oracle.conv2d(x, w, lut, layer.stride, layer.pad, q)
            G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref,
                            "%s tune %d call %d" % (layer.name, ti, call))


def test_prepare_again_with_other_filters_and_table_and_another_block():
    """A handle can be prepared again (other filters, other table) into another device block: the
    calls that follow use the new constants, the old block is left alone."""
    layer = L(2, 28, 28, 32, 3, 3, 48, 1, 1)
    x, w1, q = I.make_operands(layer, 7301)
    w2 = I.make_operands(layer, 7302)[1]
    lut1, lut2 = I.lut_truncated(5), I.lut_random(9)
    desc = ax._conv_desc(x.shape, w1.shape, 1, 1)
    xd = G.to_dev(x)
    with ax.AxLayer(desc, q) as h:
        p1 = torch.zeros(h.prepared_bytes, dtype=torch.uint8, device="cuda")
        p2 = torch.zeros(h.prepared_bytes, dtype=torch.uint8, device="cuda")
        h.prepare(G.to_dev(w1), ax.lut_to_device(lut1), prepared=p1)
        acc, y = h.run(xd)
        torch.cuda.synchronize()
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), *oracle.conv2d(x, w1, lut1, 1, 1, q), "first constants")
        snap = p1.clone()
        h.prepare(G.to_dev(w2), ax.lut_to_device(lut2), prepared=p2)
        acc, y = h.run(xd)
        torch.cuda.synchronize()
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), *oracle.conv2d(x, w2, lut2, 1, 1, q), "second constants")
        assert torch.equal(snap, p1)


def test_prepare_into_a_dirty_block_with_counters_and_ready_made_tables():
    """ax_layer_prepare owns everything in the prepared block: a block full of ones (arrival
    counters of shared tiles, ready-made tables) prepared twice with different filters gives the
    oracle's results both times, on two runs each."""
    layer = L(2, 28, 28, 32, 3, 3, 48, 1, 1)
    x, w1, q = I.make_operands(layer, 7311)
    w2 = I.make_operands(layer, 7312)[1]
    lut1, lut2 = I.lut_random_error(3), I.lut_truncated(4)
    desc = ax._conv_desc(x.shape, w1.shape, 1, 1)
    xd = G.to_dev(x)
    with ax.AxLayer(desc, q, tune=_tune(variant=2, split_k=3, combine=2, tables=2)) as h:
        plan = h.plan()
        assert plan["combine"] == 2 and plan["tables"] == 2 and plan["pieces"] > 0
        block = torch.full((h.prepared_bytes,), 255, dtype=torch.uint8, device="cuda")
        for w, lut in ((w1, lut1), (w2, lut2)):
            h.prepare(G.to_dev(w), ax.lut_to_device(lut), prepared=block)
            for call in range(2):
                acc, y = h.run(xd)
                torch.cuda.synchronize()
                G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), *oracle.conv2d(x, w, lut, 1, 1, q), "call %d" % call)


def test_handle_with_operator_variants_and_several_tables():
    rng = np.random.default_rng(77)
    # signed codes, dilation 2, implicit patch view (the activations are flipped per call)
    x = rng.integers(-128, 128, (2, 20, 20, 16)).astype(np.int8)
    w = rng.integers(-128, 128, (3, 3, 16, 40)).astype(np.int8)
    lut = I.lut_signed_random_error(3)
    q = I.Quant(0.02, -7, 0.004, 5, None)
    desc = ax._conv_desc(x.shape, w.shape, 1, 2, dilation=2, signed=True)
    with ax.AxLayer(desc, q, tune=_tune(variant=2)) as h:
        h.prepare(G.to_dev(w), ax.lut_to_device(lut))
        for call in range(2):
            acc, y = h.run(G.to_dev(x))
            torch.cuda.synchronize()
            ref = oracle.conv2d_ex(x, w, lut, 1, 2, q, dilation=2, signed=True)
            G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref[0], ref[1], "signed dilated call %d" % call)
            x = rng.integers(-128, 128, x.shape).astype(np.int8)
    # depthwise: the handle keeps the filter and table pointers, nothing is prepared
    x = rng.integers(0, 256, (2, 40, 40, 32)).astype(np.uint8)
    w = rng.integers(0, 256, (3, 3, 32, 1)).astype(np.uint8)
    lut = I.lut_random_error(5)
    q = I.Quant(0.02, 3, 0.01, 128, None)
    desc = ax._conv_desc(x.shape, w.shape, 1, 1, depthwise=True)
    with ax.AxLayer(desc, q) as h:
        assert h.prepared_bytes == 0 and h.workspace_bytes == 0
        h.prepare(G.to_dev(w), ax.lut_to_device(lut))
        acc, y = h.run(G.to_dev(x))
        torch.cuda.synchronize()
        ref = oracle.conv2d_ex(x, w, lut, 1, 1, q, depthwise=True)
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref[0], ref[1], "depthwise")
    # four tables in one handle
    layer = L(2, 14, 14, 64, 3, 3, 96, 1, 1)
    x, w, q = I.make_operands(layer, 7400)
    tabs = [np.ascontiguousarray(I.lut_random_error(s)).reshape(-1) for s in range(4)]
    desc = ax._conv_desc(x.shape, w.shape, 1, 1)
    with ax.AxLayer(desc, q, num_luts=4) as h:
        h.prepare(G.to_dev(w), torch.stack([ax.lut_to_device(t) for t in tabs]))
        acc, y = h.run(G.to_dev(x))
        torch.cuda.synchronize()
        for t in range(4):
            ref = oracle.conv2d(x, w, tabs[t], 1, 1, q)
            G.assert_parity(acc[t].cpu().numpy(), y[t].cpu().numpy(), ref[0], ref[1], "table %d" % t)


def test_kernel_timing_probe_leaves_the_results_in_place():
    layer = L(4, 28, 28, 64, 3, 3, 64, 1, 1)
    x, w, q = I.make_operands(layer, 7500)
    lut = I.lut_truncated(6)
    desc = ax._conv_desc(x.shape, w.shape, 1, 1)
    with ax.AxLayer(desc, q, tune=_tune(variant=2, split_k=2)) as h:
        h.prepare(G.to_dev(w), ax.lut_to_device(lut))
        acc = torch.empty(h.out_shape(), dtype=torch.int32, device="cuda")
        y = torch.empty(h.out_shape(), dtype=torch.float32, device="cuda")
        ms = h.kernel_ms(G.to_dev(x), acc, y, reps=3)
        assert 0.0 < ms < 50.0
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), *oracle.conv2d(x, w, lut, 1, 1, q), "after the probe")
        with pytest.raises(ax.AxError):
            h.kernel_ms(G.to_dev(x), acc, y, reps=0)


def test_run_before_prepare_is_an_error():
    desc = ax._conv_desc((2, 28, 28, 64), (3, 3, 64, 64), 1, 1)
    with ax.AxLayer(desc, I.Quant(1.0, 0, 1.0, 0, None)) as h:
        with pytest.raises(ax.AxError) as e:
            h.run(torch.zeros((2, 28, 28, 64), dtype=torch.uint8, device="cuda"))
        assert e.value.code == -9


def test_materialized_operand_beyond_four_gib():
    """Cin = 24 is no multiple of 16, so the patches are materialized: 150 x 360 x 360 pixels of
    224 padded taps are 4.35 GB, past what a 32-bit byte offset reaches.  The last image lies
    wholly beyond 2^32 and is compared with the oracle, as is the first."""
    rng = np.random.default_rng(4096)
    N, H, W, Cin, Cout = 150, 360, 360, 24, 8
    x = rng.integers(0, 256, (N, H, W, Cin), dtype=np.uint8)
    w = rng.integers(0, 256, (3, 3, Cin, Cout), dtype=np.uint8)
    lut = I.lut_truncated(6)
    q = I.Quant(0.02, 3, 0.01, 128, -1)
    acc, y = ax.ax_conv2d(G.to_dev(x), G.to_dev(w), ax.lut_to_device(lut), 1, 1, q)
    torch.cuda.synchronize()
    assert N * H * W * 224 > 1 << 32 and (N - 1) * H * W * 224 > 1 << 32
    for n in (0, N - 1):
        acc_ref, y_ref = oracle.conv2d(x[n:n + 1], w, lut, 1, 1, q)
        G.assert_parity(acc[n:n + 1].cpu().numpy(), y[n:n + 1].cpu().numpy(), acc_ref, y_ref, "image %d" % n)
