"""Pins for the multiplier-table generators and the shape lists (CPU only)."""

import numpy as np
import pytest

from paper_2002_09481_amd import inputs as I


def _t(t):
    return I.lut_truncated(t).reshape(256, 256).astype(np.int64)


def test_exact_table():
    e = I.lut_exact().reshape(256, 256)
    assert e[255, 255] == 65025 and e[0, 77] == 0 and e[3, 5] == 15
    assert np.array_equal(_t(0), e.astype(np.int64))
    assert int(e.astype(np.int64).sum()) == 1065369600


def test_truncated_table_closed_forms():
    # values worked out by hand from the partial-product array
    assert _t(4)[255, 255] == 64976 and _t(6)[255, 255] == 64704
    assert _t(4)[15, 15] == 176 and _t(6)[15, 15] == 64
    assert _t(4)[17, 19] == 320 and _t(6)[200, 100] == 19968
    for t in range(0, 9):
        assert _t(t)[16, 16] == 256
    # sum over the table: every partial-product bit is set in a quarter of the operand pairs
    for t in (1, 4, 6, 8):
        dropped = sum(2 ** (i + j) for i in range(8) for j in range(8) if i + j < t)
        assert dropped == (t - 1) * 2 ** t + 1
        assert int(_t(t).sum()) == 16384 * (65025 - dropped)
    assert int(_t(4).sum()) == 1064566784 and int(_t(6).sum()) == 1060110336


def test_truncated_error_bound_and_not_a_mask():
    e = I.lut_exact().reshape(256, 256).astype(np.int64)
    for t in (4, 6):
        d = e - _t(t)
        assert d.min() == 0 and d.max() == (t - 1) * 2 ** t + 1
        assert abs(d.mean() - ((t - 1) * 2 ** t + 1) / 4.0) < 1e-9
    assert np.count_nonzero(_t(4) != (e & ~15)) == 20224
    assert np.count_nonzero(_t(6) != (e & ~63)) == 37296


def test_random_error_table():
    e = I.lut_exact().astype(np.int64)
    r = I.lut_random_error(7).astype(np.int64)
    d = r - e
    inner = (e >= 64) & (e <= 65535 - 64)
    assert d[inner].min() == -64 and d[inner].max() == 64
    assert np.all(r >= 0) and np.all(r <= 65535)
    assert np.any(r.reshape(256, 256)[0] != 0)  # zero operands are perturbed too
    assert np.array_equal(r, I.lut_random_error(7).astype(np.int64))
    assert not np.array_equal(r, I.lut_random_error(8).astype(np.int64))


def test_other_tables():
    assert I.lut_zero().sum() == 0 and I.lut_const(9).min() == 9
    oh = I.lut_onehot(3, 200).reshape(256, 256)
    assert oh.sum() == 1 and oh[3, 200] == 1
    assert I.lut_first_operand().reshape(256, 256)[7, 100] == 7
    assert I.lut_second_operand().reshape(256, 256)[7, 100] == 100


def test_quantize_per_tensor():
    r = np.array([-1.0, 0.0, 0.5, 3.0])
    c, s, z = I.quantize_per_tensor(r)
    assert z == 64 and abs(s - 4.0 / 255.0) < 1e-7
    assert c[1] == z  # real zero maps exactly to the zero point
    assert np.max(np.abs(s * (c.astype(np.float64) - z) - r)) <= s / 2 + 1e-9
    c, s, z = I.quantize_per_tensor(np.array([0.0, 2.0, 6.0]))
    assert z == 0 and c[0] == 0 and c[2] == 255
    c, s, z = I.quantize_per_tensor(np.zeros(4))
    assert s == 1.0 and z == 0 and not c.any()


def test_workload_sizes():
    r50 = I.config_resnet50(32)
    assert len(r50) == 54 and sum(1 for l in r50 if not l.dense) == 53
    assert sum(l.macs for l in r50) == 130853896192
    assert sum(l.macs for l in I.config_resnet50(1)[:-1]) == 4087136256
    u = I.config_resnet50(32, unique=True)
    assert sum(l.count for l in u) == 54 and sum(l.macs * l.count for l in u) == 130853896192
    assert sum(l.macs for l in I.config_resnet8_cifar(1)) == 12238848
    assert sum(l.macs for l in I.config_lut_sweep()) == 10687086592
    assert [l.macs for l in I.config_gemm_shaped()] == [6576668672, 4294967296]
    assert I.config_single_layer()[0].macs == 147456
    assert max(l.K for l in r50) == 4608


def test_operand_distributions():
    l = I.config_resnet8_cifar(2)[1]
    x, w, q = I.make_operands(l, 2001)
    assert x.dtype == np.uint8 and x.shape == (2, 32, 32, 16) and w.shape == (3, 3, 16, 16)
    assert q.x_zp == 0 and 0.4 < np.mean(x == 0) < 0.6  # clipped ReLU: about half the codes are the zero point
    assert 100 < q.w_zp < 156
    x2, w2, q2 = I.make_operands(l, 2001)
    assert np.array_equal(x, x2) and np.array_equal(w, w2) and q == q2
