"""Pins of the CPU oracle against things other than itself (CPU only).

Each test would fail for a plausible mistake in the oracle: a transposed operand in the
table index, a wrong stride/pad/layout index, a dropped or mis-signed correction term, a
mishandled padded tap.
"""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2002_09481_amd import inputs as I

import helpers as Hh

SHAPES = [
    # N, H, W, Cin, KH, KW, Cout, stride, pad
    (1, 16, 16, 8, 3, 3, 8, 1, 1),
    (2, 9, 7, 5, 3, 3, 6, 2, 1),
    (2, 8, 8, 3, 7, 7, 4, 2, 3),
    (3, 5, 6, 16, 1, 1, 10, 1, 0),
    (1, 6, 6, 4, 1, 1, 3, 2, 0),
    (1, 4, 4, 2, 3, 3, 2, 1, 3),  # pad >= kernel: some windows are all padding
    (2, 7, 5, 3, 2, 3, 5, 3, 2),
]


def _rand(shape, seed, pad_code=-1, x_zp=None, w_zp=None):
    N, H, W, Cin, KH, KW, Cout, s, p = shape
    rng = np.random.default_rng(seed)
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    w = rng.integers(0, 256, (KH, KW, Cin, Cout)).astype(np.uint8)
    q = I.Quant(0.02, int(rng.integers(0, 256)) if x_zp is None else x_zp,
                0.005, int(rng.integers(0, 256)) if w_zp is None else w_zp, pad_code)
    return x, w, q, s, p


def _padc(q):
    return q.x_zp if q.pad_code < 0 else q.pad_code


def _sums(x, w, s, p, q):
    KH, KW, Cin, Cout = w.shape
    Sp = Hh.patches(x, KH, KW, s, p, _padc(q)).sum(axis=(3, 4, 5))
    Sf = w.astype(np.int64).sum(axis=(0, 1, 2))
    return Sp, Sf, KH * KW * Cin


@pytest.mark.parametrize("name", ["case_A", "case_B", "case_C", "case_D", "case_E", "case_F"])
def test_hand_cases(name):
    c = Hh.parse_cases(Hh.GOLDEN + "/hand_cases.txt")[name]
    x, w, lut, s, p, q, acc_ref, y_ref = Hh.case_operands(c)
    acc, y = oracle.conv2d(x, w, lut, s, p, q)
    assert np.array_equal(acc.reshape(-1).astype(np.int64), acc_ref)
    assert np.array_equal(y.reshape(-1).astype(np.float64), y_ref)


@pytest.mark.parametrize("shape", SHAPES)
def test_exact_table_is_integer_convolution(shape):
    x, w, q, s, p = _rand(shape, 11, pad_code=37)
    acc, _ = oracle.conv2d(x, w, I.lut_exact(), s, p, q)
    assert np.array_equal(acc.astype(np.int64), Hh.numpy_int_conv(x, w, s, p, 37))


@pytest.mark.parametrize("shape", SHAPES)
def test_arbitrary_table_matches_numpy_gather(shape):
    x, w, q, s, p = _rand(shape, 12)
    lut = I.lut_random(5)  # no symmetry, no structure
    acc, _ = oracle.conv2d(x, w, lut, s, p, q)
    assert np.array_equal(acc.astype(np.int64), Hh.numpy_lut_conv(x, w, lut, s, p, _padc(q)))


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_zero_table(shape):
    x, w, q, s, p = _rand(shape, 13)
    acc, y = oracle.conv2d(x, w, I.lut_zero(), s, p, q)
    assert not acc.any()
    Sp, Sf, K = _sums(x, w, s, p, q)
    corr = -q.w_zp * Sp[..., None] - q.x_zp * Sf[None, None, None, :] + K * q.x_zp * q.w_zp
    assert Hh.float_ok(y, float(np.float32(q.x_scale)) * float(np.float32(q.w_scale)) * corr)


@pytest.mark.parametrize("shape", SHAPES[:3] + SHAPES[5:6])
def test_onehot_table_counts_operand_pairs(shape):
    x, w, q, s, p = _rand(shape, 14, pad_code=200)
    x[x == 200] = 201  # only padded taps carry code 200
    x[..., 0] = 17
    w[w == 99] = 98
    w[:, :, 0, ::2] = 99
    KH, KW, Cin, Cout = w.shape
    for a0, b0 in [(17, 99), (200, 99), (200, int(w[0, 0, -1, -1]))]:
        acc, _ = oracle.conv2d(x, w, I.lut_onehot(a0, b0), s, p, q)
        xm = (Hh.patches(x, KH, KW, s, p, 200) == a0).astype(np.int64)
        wm = (w == b0).astype(np.int64)
        cnt = np.einsum("nyxhwc,hwco->nyxo", xm, wm)
        assert np.array_equal(acc.astype(np.int64), cnt)
        assert cnt.sum() > 0
    # the transposed pair must not count (unless it happens to coincide)
    acc, _ = oracle.conv2d(x, w, I.lut_onehot(99, 17), s, p, q)
    xm = (Hh.patches(x, KH, KW, s, p, 200) == 99).astype(np.int64)
    assert np.array_equal(acc.astype(np.int64), np.einsum("nyxhwc,hwco->nyxo", xm, (w == 17).astype(np.int64)))


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_asymmetric_tables_give_operand_sums(shape):
    x, w, q, s, p = _rand(shape, 15)
    Sp, Sf, K = _sums(x, w, s, p, q)
    acc, _ = oracle.conv2d(x, w, I.lut_first_operand(), s, p, q)
    assert np.array_equal(acc.astype(np.int64), np.broadcast_to(Sp[..., None], acc.shape))
    acc, _ = oracle.conv2d(x, w, I.lut_second_operand(), s, p, q)
    assert np.array_equal(acc.astype(np.int64), np.broadcast_to(Sf, acc.shape))


def test_linearity_in_the_table():
    x, w, q, s, p = _rand(SHAPES[1], 16)
    l1 = (I.lut_random(1) // 2).astype(np.uint16)
    l2 = (I.lut_random(2) // 2).astype(np.uint16)
    a1, _ = oracle.conv2d(x, w, l1, s, p, q)
    a2, _ = oracle.conv2d(x, w, l2, s, p, q)
    a12, _ = oracle.conv2d(x, w, (l1 + l2).astype(np.uint16), s, p, q)
    assert np.array_equal(a12, a1 + a2)
    ac, _ = oracle.conv2d(x, w, I.lut_const(321), s, p, q)
    assert np.all(ac == 321 * w.shape[0] * w.shape[1] * w.shape[2])


@pytest.mark.parametrize("shape", SHAPES)
def test_exact_table_equals_float64_conv_of_dequantized_tensors(shape):
    """With the exact multiplier the layer is quantize -> convolve -> dequantize (Sec. IV):
    y must equal a float64 library convolution of alpha1*(x-beta1), alpha2*(w-beta2) with zero
    padding.  This fixes every sign and coefficient of the correction terms."""
    x, w, q, s, p = _rand(shape, 17)  # pad_code = x_zp: padded taps are real zeros
    _, y = oracle.conv2d(x, w, I.lut_exact(), s, p, q)
    xs, ws = float(np.float32(q.x_scale)), float(np.float32(q.w_scale))
    xr = torch.from_numpy(xs * (x.astype(np.float64) - q.x_zp)).permute(0, 3, 1, 2)
    wr = torch.from_numpy(ws * (w.astype(np.float64) - q.w_zp)).permute(3, 2, 0, 1)
    ref = torch.nn.functional.conv2d(xr, wr, stride=s, padding=p).permute(0, 2, 3, 1).numpy()
    assert Hh.float_ok(y, ref, rtol=1e-5, atol=1e-6 + 1e-9 * np.abs(ref).max())


def test_truncated_table_within_error_bound():
    x, w, q, s, p = _rand(SHAPES[0], 18)
    K = w.shape[0] * w.shape[1] * w.shape[2]
    ae, _ = oracle.conv2d(x, w, I.lut_exact(), s, p, q)
    for t in (4, 6):
        at, _ = oracle.conv2d(x, w, I.lut_truncated(t), s, p, q)
        d = ae.astype(np.int64) - at.astype(np.int64)
        assert d.min() >= 0 and d.max() <= K * ((t - 1) * 2 ** t + 1) and d.max() > 0


def test_dense_is_matrix_product_and_1x1_conv():
    rng = np.random.default_rng(19)
    M, K, N = 7, 33, 12
    x = rng.integers(0, 256, (M, K)).astype(np.uint8)
    w = rng.integers(0, 256, (K, N)).astype(np.uint8)
    q = I.Quant(0.1, 3, 0.2, 250, -1)
    acc, y = oracle.dense(x, w, I.lut_exact(), q)
    assert np.array_equal(acc.astype(np.int64), x.astype(np.int64) @ w.astype(np.int64))
    ref = (np.float64(np.float32(0.1)) * (x.astype(np.float64) - 3)) @ (np.float64(np.float32(0.2)) * (w.astype(np.float64) - 250))
    assert Hh.float_ok(y, ref)
    lut = I.lut_random(3)
    acc, y = oracle.dense(x, w, lut, q)
    l2 = lut.reshape(256, 256).astype(np.int64)
    assert np.array_equal(acc.astype(np.int64), l2[x[:, :, None], w[None, :, :]].sum(axis=1))
    acc_c, y_c = oracle.conv2d(x.reshape(M, 1, 1, K), w.reshape(1, 1, K, N), lut, 1, 0, q)
    assert np.array_equal(acc_c.reshape(M, N), acc) and np.array_equal(y_c.reshape(M, N), y)


def test_sampled_outputs_agree_with_full_run():
    x, w, q, s, p = _rand(SHAPES[1], 20)
    lut = I.lut_random_error(4)
    acc, y = oracle.conv2d(x, w, lut, s, p, q)
    idx = np.random.default_rng(0).integers(0, acc.size, 50)
    a_s, y_s = oracle.conv2d_sample(x, w, lut, s, p, q, idx)
    assert np.array_equal(a_s, acc.reshape(-1)[idx]) and np.array_equal(y_s, y.reshape(-1)[idx])


def test_argument_errors():
    x, w, q, s, p = _rand(SHAPES[0], 21)
    with pytest.raises(RuntimeError):
        oracle.conv2d(x, w, I.lut_exact(), s, p, I.Quant(0.0, 1, 1.0, 1, -1))
    with pytest.raises(RuntimeError):
        oracle.conv2d(x, w, I.lut_exact(), s, p, I.Quant(1.0, 256, 1.0, 1, -1))
    with pytest.raises(RuntimeError):  # int32 accumulator overflow is reported, not wrapped
        oracle.dense(np.full((1, 40000), 255, np.uint8), np.full((40000, 1), 255, np.uint8), I.lut_const(65535), I.Quant())
