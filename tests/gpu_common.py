"""Shared pieces of the GPU parity tests: run a layer through the C ABI and through the
oracle on the same seeded operands and compare."""

import numpy as np
import torch

from oracle import oracle
from paper_2002_09481_amd import binding as ax
from paper_2002_09481_amd import inputs as I

RTOL, ATOL = 1e-5, 1e-6  # float outputs: |y - ref| <= 1e-5*|ref| + 1e-6 ; int32 accumulators: bit exact


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_gpu(x, w, lut, stride, pad, q, dense=False, **kw):
    xd, wd, ld = to_dev(x), to_dev(w), ax.lut_to_device(lut)
    if dense:
        acc, y = ax.ax_dense(xd.view(x.shape[0], -1), wd.view(-1, w.shape[-1]), ld, q, **kw)
    else:
        acc, y = ax.ax_conv2d(xd, wd, ld, stride, pad, q, **kw)
    torch.cuda.synchronize()
    return (None if acc is None else acc.cpu().numpy()), (None if y is None else y.cpu().numpy())


def run_oracle(x, w, lut, stride, pad, q, dense=False):
    if dense:
        return oracle.dense(x.reshape(x.shape[0], -1), w.reshape(-1, w.shape[-1]), lut, q)
    return oracle.conv2d(x, w, lut, stride, pad, q)


def assert_parity(acc, y, acc_ref, y_ref, what=""):
    acc = acc.reshape(acc_ref.shape)
    y = y.reshape(y_ref.shape)
    bad = np.flatnonzero(acc.reshape(-1) != acc_ref.reshape(-1))
    assert bad.size == 0, "%s: %d int32 accumulators differ, first at flat index %d: got %d want %d" % (
        what, bad.size, bad[0], acc.reshape(-1)[bad[0]], acc_ref.reshape(-1)[bad[0]])
    err = np.abs(y.astype(np.float64) - y_ref.astype(np.float64))
    tol = RTOL * np.abs(y_ref.astype(np.float64)) + ATOL
    worst = int(np.argmax(err - tol))
    assert np.all(err <= tol), "%s: float output off at %d: got %r want %r" % (
        what, worst, y.reshape(-1)[worst], y_ref.reshape(-1)[worst])


def check_layer(layer: I.Layer, seed: int, lut, what="", q_override=None, **kw):
    x, w, q = I.make_operands(layer, seed)
    if q_override is not None:
        q = q_override
    acc, y = run_gpu(x, w, lut, layer.stride, layer.pad, q, dense=layer.dense, **kw)
    acc_ref, y_ref = run_oracle(x, w, lut, layer.stride, layer.pad, q, dense=layer.dense)
    assert_parity(acc, y, acc_ref, y_ref, what or layer.name)
