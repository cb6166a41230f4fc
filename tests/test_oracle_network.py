"""Pins for the oracle's network glue: the residual form of the convolution and the two
pooling layers, against PyTorch CPU operators in fp64 and against their definitions."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def _nchw(a):
    return torch.from_numpy(np.ascontiguousarray(a)).double().permute(0, 3, 1, 2)


@pytest.mark.parametrize("k,stride,pad,H,W,C", [(3, 2, 1, 11, 9, 5), (2, 2, 0, 8, 8, 4), (3, 1, 1, 7, 6, 3),
                                                 (5, 3, 2, 13, 12, 2), (3, 2, 0, 7, 7, 8)])
def test_maxpool_equals_torch(k, stride, pad, H, W, C):
    rng = np.random.default_rng(k * 100 + H)
    x = rng.standard_normal((3, H, W, C)).astype(np.float32)
    got = oracle.maxpool2d(x, k, stride, pad)
    ref = F.max_pool2d(_nchw(x), k, stride, pad).permute(0, 2, 3, 1).numpy()
    assert got.shape == ref.shape
    assert np.array_equal(got, ref.astype(np.float32))


def test_maxpool_padding_never_wins():
    # all-negative input: a zero-padding implementation would return zeros at the border
    x = -np.ones((1, 4, 4, 1), dtype=np.float32) * np.arange(1, 17, dtype=np.float32).reshape(1, 4, 4, 1)
    got = oracle.maxpool2d(x, 3, 2, 1)
    assert got.max() < 0
    assert got[0, 0, 0, 0] == -1.0            # window covers rows/cols 0..1: max is x[0,0]
    assert got[0, 1, 1, 0] == x[0, 1:4, 1:4, 0].max()


def test_maxpool_rejects_bad_arguments():
    x = np.zeros((1, 4, 4, 1), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.maxpool2d(x, 3, 2, 3)          # pad >= k
    with pytest.raises(ValueError):
        oracle.maxpool2d(x, 7, 1, 1)          # window larger than the padded image


@pytest.mark.parametrize("H,W,C", [(7, 7, 16), (1, 1, 3), (5, 9, 33)])
def test_avgpool_is_the_mean(H, W, C):
    rng = np.random.default_rng(H * W + C)
    x = (rng.standard_normal((2, H, W, C)) * 3 + 1).astype(np.float32)
    got = oracle.avgpool_global(x)
    ref = x.astype(np.float64).mean(axis=(1, 2))
    assert np.allclose(got, ref, rtol=0, atol=1e-6)
    ref_t = F.adaptive_avg_pool2d(_nchw(x), 1)[:, :, 0, 0].numpy()
    assert np.allclose(got, ref_t, rtol=0, atol=1e-6)
    # constant input -> the constant, exactly
    c = np.full((1, H, W, C), 0.375, dtype=np.float32)
    assert np.array_equal(oracle.avgpool_global(c), np.full((1, C), 0.375, dtype=np.float32))


def test_avgpool_bf16_rounds_once():
    x = np.full((1, 2, 2, 1), 1.0, dtype=np.float32)
    x[0, 0, 0, 0] = 1.0 + 2.0 ** -6           # mean = 1 + 2^-8: a tie between 1 and 1 + 2^-7 -> even (1.0)
    assert oracle.avgpool_global(x, out_bf16=True)[0, 0] == 1.0
    assert oracle.avgpool_global(x)[0, 0] == np.float32(1.0 + 2.0 ** -8)


@pytest.mark.parametrize("stride,pad,dil,relu", [(1, 1, 1, True), (2, 1, 1, False), (1, 2, 2, True), (1, 0, 1, True)])
def test_residual_conv_equals_torch(stride, pad, dil, relu):
    rng = np.random.default_rng(stride * 10 + pad)
    x = rng.standard_normal((2, 9, 8, 6)).astype(np.float32)
    w = rng.standard_normal((10, 3, 3, 6)).astype(np.float32)
    b = rng.standard_normal(10).astype(np.float32)
    plain = oracle.conv2d(x, w, b, stride, pad, dil, False)
    r = rng.standard_normal(plain.shape).astype(np.float32)
    got = oracle.conv2d_res(x, w, r, b, stride, pad, dil, relu)
    t = F.conv2d(_nchw(x), torch.from_numpy(w).double().permute(0, 3, 1, 2), torch.from_numpy(b).double(),
                 stride, pad, dil) + _nchw(r)
    if relu:
        t = F.relu(t)
    ref = t.permute(0, 2, 3, 1).numpy()
    assert np.allclose(got, ref, rtol=0, atol=2e-6 * (1 + np.abs(ref).max()))


def test_residual_is_added_before_the_activation_and_zero_residual_changes_nothing():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 5, 5, 4)).astype(np.float32)
    w = rng.standard_normal((3, 3, 3, 4)).astype(np.float32)
    plain = oracle.conv2d(x, w, None, 1, 1, 1, False)
    zero = np.zeros_like(plain)
    assert np.array_equal(oracle.conv2d_res(x, w, zero, None, 1, 1, 1, True), oracle.conv2d(x, w, None, 1, 1, 1, True))
    # residual = -conv - 1 makes every pre-activation exactly -1 -> relu gives 0; relu(conv) + residual would not
    r = -plain - 1.0
    assert np.array_equal(oracle.conv2d_res(x, w, r, None, 1, 1, 1, True), zero)
    got = oracle.conv2d_res(x, w, r, None, 1, 1, 1, False)
    assert np.allclose(got, -1.0, atol=1e-5)
    with pytest.raises(ValueError):
        oracle.conv2d_res(x, w, zero[:, :-1], None, 1, 1, 1, True)


@pytest.mark.parametrize("kh,kw,stride,pad,dil", [(3, 3, 1, 1, 1), (3, 3, 2, 1, 1), (1, 1, 2, 0, 1), (5, 3, 1, 2, 2), (7, 7, 2, 3, 1)])
def test_im2col_equals_unfold_and_turns_the_convolution_into_a_matrix_product(kh, kw, stride, pad, dil):
    rng = np.random.default_rng(kh * 7 + stride)
    x = rng.standard_normal((2, 11, 10, 3)).astype(np.float32)
    a = oracle.im2col(x, kh, kw, stride, pad, dil)
    # torch.unfold orders k as (ci, kh, kw); reorder to (kh, kw, ci)
    u = F.unfold(_nchw(x), (kh, kw), dilation=dil, padding=pad, stride=stride)        # [B, C*kh*kw, L]
    B, _, Lp = u.shape
    u = u.reshape(B, 3, kh, kw, Lp).permute(0, 4, 2, 3, 1).reshape(B, Lp, kh * kw * 3).numpy()
    assert np.array_equal(a.reshape(B, Lp, -1), u.astype(np.float32))
    w = rng.standard_normal((4, kh, kw, 3)).astype(np.float32)
    y = oracle.conv2d(x, w, None, stride, pad, dil, False)
    ref = a.reshape(B, Lp, -1).astype(np.float64) @ w.reshape(4, -1).astype(np.float64).T
    assert np.allclose(y.reshape(B, Lp, 4), ref, rtol=0, atol=1e-5)
    # and a 1x1 convolution over the im2col tensor is the original convolution
    y1 = oracle.conv2d(a, w.reshape(4, 1, 1, -1), None, 1, 0, 1, False)
    assert np.array_equal(y1, y)
