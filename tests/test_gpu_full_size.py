"""GPU parity at the full sizes of the five workloads, in the launch configurations that
bench.py times: layer handles with filters and table prepared once (automatic variant / tile /
work decomposition), and the one-call entry points beside them.

Every output of every distinct layer shape is compared with the oracle, element by element
(bit-exact int32, 1e-5*|ref| + 1e-6 for the float outputs): the planner's full-size choices
(balanced tile heights, XCD numbering of the shares, grids with partial pieces and the fix-up
pass, the vectorized epilogue) only occur at these sizes.  The one exception is the 64-table
sweep, where the oracle does tables 0, 31 and 63 whole and sampled outputs of the other 61
(all 64 whole would be 0.7 T lookups on the host, minutes of a GPU machine's time).
"""

import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu

SAMPLES = 384


def _desc(layer):
    if layer.dense:
        return ax._dense_desc(layer.N, layer.K, layer.Cout)
    return ax._conv_desc((layer.N, layer.H, layer.W, layer.Cin), (layer.KH, layer.KW, layer.Cin, layer.Cout),
                         layer.stride, layer.pad)


def _run(layer, x, w, lut_d, q):
    """One-call entry points (table re-laid out and filters packed inside the call)."""
    xd, wd = G.to_dev(x), G.to_dev(w)
    if layer.dense:
        acc, y = ax.ax_dense(xd.view(layer.N, layer.K), wd.view(layer.K, layer.Cout), lut_d, q)
    else:
        acc, y = ax.ax_conv2d(xd, wd, lut_d, layer.stride, layer.pad, q)
    torch.cuda.synchronize()
    return acc, y


def _run_handle(layer, x, w, lut_d, q, calls=1):
    """Layer handle: prepare once, run `calls` times (the last call's results are returned)."""
    xd, wd = G.to_dev(x), G.to_dev(w)
    with ax.AxLayer(_desc(layer), q) as h:
        h.prepare(wd, lut_d)
        for _ in range(calls):
            acc, y = h.run(xd)
        torch.cuda.synchronize()
        plan = h.plan()
    return acc, y, plan


def _oracle(layer, x, w, lut, q):
    if layer.dense:
        return oracle.dense(x.reshape(layer.N, layer.K), w.reshape(layer.K, layer.Cout), lut, q)
    return oracle.conv2d(x, w, lut, layer.stride, layer.pad, q)


def _check_whole(layer, x, w, lut, q, acc, y, what):
    acc_ref, y_ref = _oracle(layer, x, w, lut, q)
    G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, what)


def _check_sampled(layer, x, w, lut, q, acc, y, rng, what):
    n_out = layer.M * layer.Cout
    # random outputs plus the corners of the tensor (first / last pixel and channel)
    idx = np.concatenate([rng.integers(0, n_out, size=SAMPLES),
                          np.array([0, layer.Cout - 1, n_out - layer.Cout, n_out - 1])]).astype(np.int64)
    a_ref, y_ref = oracle.conv2d_sample(x, w, lut, layer.stride, layer.pad, q, idx)
    ti = torch.from_numpy(idx).cuda()
    a_g = acc.reshape(-1)[ti].cpu().numpy()
    y_g = y.reshape(-1)[ti].cpu().numpy()
    G.assert_parity(a_g, y_g, a_ref, y_ref, what)


def test_config2_full_batch_elementwise():
    lut = I.lut_random_error(2000)
    lut_d = ax.lut_to_device(lut)
    for i, layer in enumerate(I.config_resnet8_cifar(batch=128)):
        x, w, q = I.make_operands(layer, I.layer_seed(2, i))
        acc, y = _run(layer, x, w, lut_d, q)
        acc_ref, y_ref = oracle.conv2d(x, w, lut, layer.stride, layer.pad, q)
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, layer.name)


def test_config3_resnet50_batch32_every_output_of_every_shape():
    """All 24 distinct layer shapes of the ResNet-50-shaped workload at batch 32: the prepared
    handle (second of two calls, as in a timed loop) against the oracle on every output, the
    one-call entry against the handle bit for bit, and a constant table through both."""
    lut = I.lut_truncated(6)
    lut_d = ax.lut_to_device(lut)
    const_d = ax.lut_to_device(I.lut_const(3))
    layers = I.config_resnet50(32)
    seen = set()
    with_pieces = 0
    for i, layer in enumerate(layers):
        key = (layer.H, layer.Cin, layer.KH, layer.Cout, layer.stride, layer.dense)
        if key in seen:
            continue
        seen.add(key)
        x, w, q = I.make_operands(layer, I.layer_seed(3, i))
        acc, y, plan = _run_handle(layer, x, w, lut_d, q, calls=2)
        with_pieces += plan["pieces"] > 0
        _check_whole(layer, x, w, lut, q, acc, y, layer.name)
        acc1, y1 = _run(layer, x, w, lut_d, q)
        assert torch.equal(acc1.reshape(-1), acc.reshape(-1)) and torch.equal(y1.reshape(-1), y.reshape(-1)), \
            "%s: one-call entry and prepared handle differ" % layer.name
        acc_c, _ = _run(layer, x, w, const_d, q)
        assert bool((acc_c == 3 * layer.K).all()), "%s: constant table must give c*K everywhere" % layer.name
    assert len(seen) == 24
    assert with_pieces >= 1  # the sweep exercises the fix-up pass at full size


def test_config4_lut_sweep_layers_batch64_three_tables_whole():
    for i, layer in enumerate(I.config_lut_sweep(batch=64)):
        x, w, q = I.make_operands(layer, I.layer_seed(4, i))
        for lut_seed in (0, 31, 63):
            lut = I.lut_random_error(lut_seed)
            acc, y = _run(layer, x, w, ax.lut_to_device(lut), q)
            _check_whole(layer, x, w, lut, q, acc, y, "%s lut %d" % (layer.name, lut_seed))


def test_config4_all_64_tables_one_call_per_layer():
    """Both layers of the table sweep at batch 64 against all 64 tables (one multi-table call per
    layer): tables 0, 31 and 63 compared whole, a handful of outputs of each of the others checked
    one by one by the oracle."""
    rng = np.random.default_rng(464)
    tabs = [np.ascontiguousarray(I.lut_random_error(sd)).reshape(-1) for sd in range(64)]
    luts_d = torch.stack([ax.lut_to_device(t) for t in tabs])
    for i, layer in enumerate(I.config_lut_sweep(batch=64)):
        x, w, q = I.make_operands(layer, I.layer_seed(4, i))
        acc, y = ax.ax_conv2d_multi_lut(G.to_dev(x), G.to_dev(w), luts_d, layer.stride, layer.pad, q)
        torch.cuda.synchronize()
        n_out = layer.M * layer.Cout
        for t in range(64):
            if t in (0, 31, 63):
                _check_whole(layer, x, w, tabs[t], q, acc[t], y[t], "%s table %d" % (layer.name, t))
                continue
            idx = np.concatenate([rng.integers(0, n_out, size=24), np.array([0, n_out - 1])]).astype(np.int64)
            a_ref, y_ref = oracle.conv2d_sample(x, w, tabs[t], layer.stride, layer.pad, q, idx)
            ti = torch.from_numpy(idx).cuda()
            G.assert_parity(acc[t].reshape(-1)[ti].cpu().numpy(), y[t].reshape(-1)[ti].cpu().numpy(), a_ref, y_ref,
                            "%s table %d" % (layer.name, t))
        del acc, y


def test_config5_gemm_shaped_both_tables_whole():
    exact, trunc = I.lut_exact(), I.lut_truncated(6)
    for i, layer in enumerate(I.config_gemm_shaped()):
        x, w, q = I.make_operands(layer, I.layer_seed(5, i))
        acc, y, _ = _run_handle(layer, x, w, ax.lut_to_device(exact), q)
        # exact products -> integer GEMM (float64 on the device is exact here), and the oracle
        xm = G.to_dev(x).reshape(layer.M, layer.K).double()
        wm = G.to_dev(w).reshape(layer.K, layer.Cout).double()
        ref = (xm @ wm).to(torch.int64)
        assert torch.equal(acc.reshape(layer.M, layer.Cout).to(torch.int64), ref), layer.name
        _check_whole(layer, x, w, exact, q, acc, y, layer.name + " exact")
        acc, y, _ = _run_handle(layer, x, w, ax.lut_to_device(trunc), q)
        _check_whole(layer, x, w, trunc, q, acc, y, layer.name + " truncated")
        acc1, y1 = _run(layer, x, w, ax.lut_to_device(trunc), q)
        assert torch.equal(acc1.reshape(-1), acc.reshape(-1)) and torch.equal(y1.reshape(-1), y.reshape(-1))
        # error bound of the truncated multiplier: 0 <= exact - truncated <= K * 321
        d = ref - acc.reshape(layer.M, layer.Cout).to(torch.int64)
        assert int(d.min()) >= 0 and int(d.max()) <= layer.K * 321


def test_config3_float_layers_batch32_codes_and_outputs_whole():
    """The float-in / float-out form at full size: a stem, a 3x3, a strided 1x1 and the last
    1x1 of the ResNet-50-shaped sweep at batch 32.  Ranges, activation codes, accumulators and
    float outputs are compared whole with the float oracle."""
    lut = I.lut_truncated(6)
    lut_d = ax.lut_to_device(lut)
    layers = I.config_resnet50(32)
    picked = [0, 2, 12, 52]
    for i in picked:
        layer = layers[i]
        assert not layer.dense
        x, w = I.make_float_operands(layer, I.layer_seed(3, i))
        relu = i > 0
        xd, wd = G.to_dev(x), G.to_dev(w)
        xr, wr = ax.ax_range_f32(xd, relu=relu), ax.ax_range_f32(wd)
        if i % 4 == 0:
            acc, y = ax.ax_conv2d_f32(xd, wd, lut_d, layer.stride, layer.pad, xr, wr, relu=relu)
        else:  # ranges taken inside the layer
            acc, y = ax.ax_conv2d_f32(xd, wd, lut_d, layer.stride, layer.pad, relu=relu)
        torch.cuda.synchronize()
        xr_o, wr_o = oracle.range_f32(x, relu), oracle.range_f32(w)
        np.testing.assert_array_equal(xr.cpu().numpy(), xr_o)
        np.testing.assert_array_equal(wr.cpu().numpy(), wr_o)
        ref = oracle.conv2d_f32(x, w, lut, layer.stride, layer.pad, xr_o, wr_o, relu=relu)
        codes, _ = ax.ax_quantize_f32(xd, xr, relu=relu)
        assert bool((codes == G.to_dev(ref["xq"])).all()), "%s: activation codes differ" % layer.name
        G.assert_parity(acc.cpu().numpy(), y.cpu().numpy(), ref["acc"], ref["y"], layer.name + " (float)")
