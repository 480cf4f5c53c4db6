"""The layer calls only enqueue kernels (no allocation, no synchronization, no memset), so a
sequence of them can be captured into a HIP graph.  Every replay must reproduce the eager result,
also with the library's own eager work and synchronizations between the replays."""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

import gpu_common as G

pytestmark = pytest.mark.gpu


def test_captured_stack_replays_match_eager_and_oracle():
    layers = I.config_resnet8_cifar(batch=8)
    lut = I.lut_random_error(2000)
    lut_d = ax.lut_to_device(lut)
    calls, host = [], []
    for i, l in enumerate(layers):
        x, w, q = I.make_operands(l, I.layer_seed(2, i))
        xd, wd = G.to_dev(x), G.to_dev(w)
        acc = torch.zeros((l.N, l.OH, l.OW, l.Cout), dtype=torch.int32, device="cuda")
        y = torch.zeros(acc.shape, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(256, ax.ax_conv2d_workspace_bytes(x.shape, w.shape, l.stride, l.pad)), dtype=torch.uint8,
                         device="cuda")
        calls.append((l, xd, wd, q, acc, y, ws))
        host.append((x, w, q))
    # one float layer (ranges taken inside the call) rides along
    fl = layers[3]
    xf, wf = I.make_float_operands(fl, 77)
    xfd, wfd = G.to_dev(xf), G.to_dev(wf)
    facc = torch.zeros((fl.N, fl.OH, fl.OW, fl.Cout), dtype=torch.int32, device="cuda")
    fy = torch.zeros(facc.shape, dtype=torch.float32, device="cuda")
    fws = torch.empty(ax.ax_conv2d_f32_workspace_bytes(xf.shape, wf.shape, fl.stride, fl.pad), dtype=torch.uint8,
                      device="cuda")

    def step():
        for l, xd, wd, q, acc, y, ws in calls:
            ax.ax_conv2d(xd, wd, lut_d, l.stride, l.pad, q, acc, y, ws)
        ax.ax_conv2d_f32(xfd, wfd, lut_d, fl.stride, fl.pad, None, None, True, 0, facc, fy, fws)

    step()
    torch.cuda.synchronize()
    eager = [(c[4].clone(), c[5].clone()) for c in calls] + [(facc.clone(), fy.clone())]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    outs = [(c[4], c[5]) for c in calls] + [(facc, fy)]
    for rep in range(3):
        for a, y in outs:  # eager work between the replays: wipe the outputs
            a.zero_()
            y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (a, y), (ea, ey) in zip(outs, eager):
            assert torch.equal(a, ea) and torch.equal(y, ey), "replay %d differs from the eager run" % rep
    for (l, *_), (x, w, q), (a, y) in zip(calls, host, eager):
        acc_ref, y_ref = oracle.conv2d(x, w, lut, l.stride, l.pad, q)
        G.assert_parity(a.cpu().numpy(), y.cpu().numpy(), acc_ref, y_ref, l.name)
