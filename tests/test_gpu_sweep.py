"""Table sweeps with the upload of the next tables overlapping the layers that run on the
current ones (paper_2002_09481_amd.sweep.TableSweep): the results must equal, bit for bit,
those of the same layers on tables that were resident in device memory all along, and the
oracle's."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I
from paper_2002_09481_amd.sweep import TableSweep

import gpu_common as G

pytestmark = pytest.mark.gpu


def _layers():
    out = []
    for i, l in enumerate((I.Layer("sw.a", 4, 28, 28, 64, 1, 1, 48, 1, 0, x_dist="relu", w_dist="normal"),
                           I.Layer("sw.b", 4, 28, 28, 32, 3, 3, 48, 1, 1, x_dist="uniform", w_dist="uniform"),
                           I.Layer("sw.tiny", 1, 6, 6, 4, 3, 3, 5, 1, 1))):  # direct kernel: reads the table in every call
        x, w, q = I.make_operands(l, 8800 + i)
        out.append((l, x, w, q))
    return out


@pytest.mark.parametrize("chunk,per_upload", [(1, 1), (1, 3), (2, 2), (2, 4), (4, None)])
def test_overlapped_sweep_equals_resident_tables(chunk, per_upload):
    T = 7
    tabs = [np.ascontiguousarray(I.lut_random_error(300 + t)).reshape(-1) for t in range(T)]
    host = torch.from_numpy(np.stack(tabs).view(np.int16).copy()).pin_memory()
    layers = _layers()
    dev_layers = [(ax._conv_desc(x.shape, w.shape, l.stride, l.pad), q, G.to_dev(x), G.to_dev(w))
                  for l, x, w, q in layers]
    sweep = TableSweep(dev_layers, chunk=chunk, tables_per_upload=per_upload)
    try:
        for rnd in range(2):  # the second round reuses staging buffers, blocks and events
            acc, y = sweep.run(host, overlap=True)
            acc_s, y_s = sweep.run(host, overlap=False)
            torch.cuda.synchronize()
            for li, (l, x, w, q) in enumerate(layers):
                # resident tables, one plain call per table
                for t in range(T):
                    a_r, y_r = ax.ax_conv2d(G.to_dev(x), G.to_dev(w), ax.lut_to_device(tabs[t]), l.stride, l.pad, q)
                    torch.cuda.synchronize()
                    assert torch.equal(acc[li][t], a_r) and torch.equal(y[li][t], y_r), (l.name, t, rnd)
                    assert torch.equal(acc_s[li][t], a_r) and torch.equal(y_s[li][t], y_r), (l.name, t, rnd)
                a_ref, y_ref = oracle.conv2d(x, w, tabs[T - 1], l.stride, l.pad, q)
                G.assert_parity(acc[li][T - 1].cpu().numpy(), y[li][T - 1].cpu().numpy(), a_ref, y_ref, l.name)
    finally:
        sweep.close()
