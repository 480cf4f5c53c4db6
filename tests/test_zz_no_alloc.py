"""The allocation-free entry point ax_layer_run_static (scratch in a static device array of the
library) against ax_layer_run (caller workspace): same bits, on two calls in a row, the second
with a smaller input, for layers whose kernels really use the scratch (materialized patches,
pieces of shared tiles and the fix-up pass, packed patches for channel lanes)."""

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


def _layer(N, H, W, Cin, KH, KW, Cout, s, p):
    return I.Layer("s%dx%dx%dx%d_k%d_c%d" % (N, H, W, Cin, KH, Cout), N, H, W, Cin, KH, KW, Cout, s, p,
                   x_dist="relu", w_dist="normal")


# (first call, second and smaller call, tune)
CASES = [
    # materialized patches (Cin % 16 != 0) and K slices: pieces + fix-up pass
    (_layer(4, 40, 40, 20, 3, 3, 48, 1, 1), _layer(2, 24, 24, 20, 3, 3, 48, 1, 1), _tune(variant=2, split_k=3)),
    # channel lanes: packed patches and their sums live in the scratch
    (_layer(2, 14, 14, 128, 3, 3, 600, 1, 1), _layer(1, 9, 9, 128, 3, 3, 600, 1, 1), _tune(variant=3, split_k=2)),
    # automatic plan of a layer with few pixels and a long sum (K slices at full machine width)
    (_layer(8, 7, 7, 512, 3, 3, 512, 1, 1), _layer(4, 7, 7, 512, 3, 3, 512, 1, 1), _tune()),
    # activations read in place, no pieces: the call needs no scratch at all
    (_layer(8, 28, 28, 64, 3, 3, 64, 1, 1), _layer(2, 28, 28, 64, 3, 3, 64, 1, 1), _tune()),
]


@pytest.mark.parametrize("ci", range(len(CASES)))
def test_static_scratch_entry_matches_workspace_entry_on_two_calls(ci):
    first, second, tune = CASES[ci]
    lut = I.lut_random_error(90 + ci)
    lut_d = ax.lut_to_device(lut)
    for call, layer in enumerate((first, second)):
        x, w, q = I.make_operands(layer, 9000 + 10 * ci + (0 if call == 0 else 1))
        if call == 1:  # same filters for both calls of a case: only the activations' shape shrinks
            w = I.make_operands(first, 9000 + 10 * ci)[1]
        desc = ax._conv_desc(x.shape, w.shape, layer.stride, layer.pad)
        xd, wd = G.to_dev(x), G.to_dev(w)
        with ax.AxLayer(desc, q, tune=tune) as h:
            h.prepare(wd, lut_d)
            acc_ws, y_ws = h.run(xd)
            acc_st = torch.full(h.out_shape(), -1, dtype=torch.int32, device="cuda")
            y_st = torch.full(h.out_shape(), float("nan"), dtype=torch.float32, device="cuda")
            h.run_static(xd, acc_st, y_st)
            torch.cuda.synchronize()
            assert torch.equal(acc_st, acc_ws), "case %d call %d: accumulators differ" % (ci, call)
            assert torch.equal(y_st, y_ws), "case %d call %d: float outputs differ" % (ci, call)
            acc_ref, y_ref = oracle.conv2d(x, w, lut, layer.stride, layer.pad, q)
            G.assert_parity(acc_st.cpu().numpy(), y_st.cpu().numpy(), acc_ref, y_ref, "case %d call %d" % (ci, call))


def test_static_scratch_limit_and_state_errors():
    limit = ax.ax_static_scratch_bytes()
    assert limit == 64 << 20
    # a layer whose pieces need more scratch than the array holds is refused, nothing is launched
    big = ax._conv_desc((32, 14, 14, 1024), (1, 1, 1024, 512), 1, 0)
    q = I.Quant(0.02, 3, 0.01, 128, -1)
    with ax.AxLayer(big, q, tune=_tune(variant=2, split_k=8, tile=3)) as h:
        assert h.workspace_bytes > limit
        x = torch.zeros((32, 14, 14, 1024), dtype=torch.uint8, device="cuda")
        acc = torch.empty(h.out_shape(), dtype=torch.int32, device="cuda")
        with pytest.raises(ax.AxError) as e:  # not prepared
            h.run_static(x, acc, False)
        assert e.value.code == -9
        h.prepare(torch.zeros((1, 1, 1024, 512), dtype=torch.uint8, device="cuda"),
                  ax.lut_to_device(I.lut_exact()))
        with pytest.raises(ax.AxError) as e:
            h.run_static(x, acc, False)
        assert e.value.code == -5
    torch.cuda.synchronize()


def test_static_entry_under_graph_capture_replays_like_eager_calls():
    """What the allocation-free entry point is for: three layers (materialized patches with a
    fix-up pass, shared tiles combined inside the main kernel, activations read in place) recorded
    once into a HIP graph and replayed on new activations.  Every replay is compared with eager
    calls on the same activations, with eager work of the library between the replays."""
    cases = [(CASES[0][0], CASES[0][2]), (_layer(8, 7, 7, 512, 3, 3, 512, 1, 1), _tune(variant=2, split_k=2, combine=2)),
             (CASES[3][0], CASES[3][2])]
    lut_d = ax.lut_to_device(I.lut_random_error(97))
    hs = []
    for i, (layer, tune) in enumerate(cases):
        x, w, q = I.make_operands(layer, 9100 + i)
        h = ax.AxLayer(ax._conv_desc(x.shape, w.shape, layer.stride, layer.pad), q, tune=tune)
        h.prepare(G.to_dev(w), lut_d)
        xd = G.to_dev(x)
        acc = torch.empty(h.out_shape(), dtype=torch.int32, device="cuda")
        y = torch.empty(h.out_shape(), dtype=torch.float32, device="cuda")
        hs.append((layer, h, xd, acc, y))
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):  # once eagerly on the capture stream, as torch asks
            for layer, h, xd, acc, y in hs:
                h.run_static(xd, acc, y)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for layer, h, xd, acc, y in hs:
                h.run_static(xd, acc, y)
        torch.cuda.synchronize()
        for rep in range(3):
            for i, (layer, h, xd, acc, y) in enumerate(hs):  # new activations in the recorded buffers
                xd.copy_(G.to_dev(I.make_operands(layer, 9200 + 10 * rep + i)[0]))
                acc.fill_(-1)
                y.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            for i, (layer, h, xd, acc, y) in enumerate(hs):
                acc_e, y_e = h.run(xd)  # eager, caller workspace
                torch.cuda.synchronize()
                assert torch.equal(acc, acc_e), "replay %d layer %d: accumulators differ" % (rep, i)
                assert torch.equal(y, y_e), "replay %d layer %d: float outputs differ" % (rep, i)
    finally:
        for _, h, _, _, _ in hs:
            h.close()
    torch.cuda.synchronize()
