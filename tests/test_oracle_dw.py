"""Pins for the oracle's weight gradients (FC and conv).

Checked against: hand-computed integer examples, the fp64 library matmul /
library conv-weight-gradient, an independent explicit-im2col formulation, the
paper's split identity (full gradient = dropped part + retained part, Sec. 3.2
Eq. conv_backward_elem_split), gamma = 0 reproducing the dense gradient, the
1x1-conv == FC special case, and the closed form for a single retained element.
"""
import numpy as np
import pytest
import torch

import oracle
from dropit_inputs import activation, gradient


# ---------------------------------------------------------------- FC
def test_fc_hand_computed():
    # 3 tokens, cin = 2, cout = 2:  dW[j][c] = sum_n dY[n][j] * x[n][c]
    x = np.array([[1.0, 2.0], [0.0, -1.0], [3.0, 0.0]])
    dy = np.array([[1.0, 10.0], [2.0, 20.0], [-1.0, 5.0]])
    # dW[0][0] = 1*1 + 2*0 + (-1)*3 = -2 ; dW[0][1] = 1*2 + 2*(-1) + 0 = 0
    # dW[1][0] = 10*1 + 0 + 5*3 = 25     ; dW[1][1] = 10*2 + 20*(-1) + 0 = 0
    assert np.array_equal(oracle.dw_fc(x, dy), np.array([[-2.0, 0.0], [25.0, 0.0]]))


def test_fc_shape_is_cout_by_cin_and_not_transposed():
    x = np.zeros((4, 3))
    dy = np.zeros((4, 5))
    x[2, 1] = 2.0
    dy[2, 4] = 7.0
    dW = oracle.dw_fc(x, dy)
    assert dW.shape == (5, 3)
    want = np.zeros((5, 3))
    want[4, 1] = 14.0
    assert np.array_equal(dW, want)


def test_fc_equals_library_matmul_fp64():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((97, 33))
    dy = rng.standard_normal((97, 21))
    np.testing.assert_allclose(oracle.dw_fc(x, dy), dy.T @ x, rtol=0, atol=1e-12)
    # row-range form returns the same rows
    np.testing.assert_array_equal(oracle.dw_fc(x, dy, 5, 9), oracle.dw_fc(x, dy)[5:9])


def test_fc_leading_dims_are_tokens():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 5, 7))
    dy = rng.standard_normal((2, 5, 3))
    np.testing.assert_allclose(oracle.dw_fc(x, dy), dy.reshape(10, 3).T @ x.reshape(10, 7), atol=1e-13)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fc_gamma_zero_is_dense_and_split_identity(dtype):
    x = activation((128, 48), "normal", 11, dtype)
    dy = gradient((128, 24), 0.02, 12, dtype)
    xw, dyw = oracle.widen(x), oracle.widen(dy)
    dense = oracle.dw_fc(xw, dyw)
    # gamma = 0: keep everything -> exactly the dense gradient
    vals, idx = oracle.compress(x, x.size)
    assert np.array_equal(oracle.dw_fc(oracle.densify(vals, idx, x.shape), dyw), dense)
    # split identity: dW(x) = dW(x_hat) + dW(x - x_hat)
    k = oracle.keep_count(x.size, 0.9)
    vals, idx = oracle.compress(x, k)
    xh = oracle.densify(vals, idx, x.shape)
    np.testing.assert_allclose(oracle.dw_fc(xh, dyw) + oracle.dw_fc(xw - xh, dyw), dense,
                               rtol=0, atol=1e-12 * np.abs(dense).max())
    # and dropping really changed something
    assert np.count_nonzero(xh) <= k < x.size


def test_fc_statistics_of_retained_energy():
    # N(0,1) input, gamma=.9: retained second moment 2[t*phi(t) + 0.05] = 0.4393 at t = 1.6449,
    # so std(dW) ~ 0.02 * sqrt(ntok * 0.4393)
    ntok = 4096
    x = activation((ntok, 64), "normal", 21, "bf16")
    dy = gradient((ntok, 32), 0.02, 22, "bf16")
    k = oracle.keep_count(x.size, 0.9)
    vals, idx = oracle.compress(x, k)
    dW = oracle.dw_fc(oracle.densify(vals, idx, x.shape), oracle.widen(dy))
    expect = 0.02 * np.sqrt(ntok * 0.4393)
    assert abs(dW.std() / expect - 1.0) < 0.06


# ---------------------------------------------------------------- conv
def im2col_dw(x, dy, kh, kw, stride, pad, dil):
    """Independent formulation: explicit im2col matrix, then one matmul."""
    N, C, H, W = x.shape
    _, J, OH, OW = dy.shape
    cols = np.zeros((N, OH, OW, C, kh, kw))
    for u in range(kh):
        for v in range(kw):
            for oy in range(OH):
                iy = oy * stride[0] - pad[0] + u * dil[0]
                if not 0 <= iy < H:
                    continue
                for ox in range(OW):
                    ix = ox * stride[1] - pad[1] + v * dil[1]
                    if 0 <= ix < W:
                        cols[:, oy, ox, :, u, v] = x[:, :, iy, ix]
    A = dy.transpose(1, 0, 2, 3).reshape(J, N * OH * OW)
    return (A @ cols.reshape(N * OH * OW, C * kh * kw)).reshape(J, C, kh, kw)


def _out_hw(H, W, kh, kw, s, p, d):
    return ((H + 2 * p[0] - d[0] * (kh - 1) - 1) // s[0] + 1,
            (W + 2 * p[1] - d[1] * (kw - 1) - 1) // s[1] + 1)


CONV_CASES = [
    # N, C, H, W, J, kh, kw, stride, pad, dil
    (2, 3, 8, 8, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 3, 9, 7, 2, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 2, 10, 11, 3, 3, 2, (1, 2), (0, 1), (2, 1)),
    (2, 4, 6, 6, 5, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 1, 16, 16, 2, 7, 7, (2, 2), (3, 3), (1, 1)),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_equals_im2col_and_library(case):
    N, C, H, W, J, kh, kw, s, p, d = case
    rng = np.random.default_rng(hash(case) % 2**32)
    OH, OW = _out_hw(H, W, kh, kw, s, p, d)
    x = rng.standard_normal((N, C, H, W))
    dy = rng.standard_normal((N, J, OH, OW))
    got = oracle.dw_conv(x, dy, kh, kw, s, p, d)
    np.testing.assert_allclose(got, im2col_dw(x, dy, kh, kw, s, p, d), rtol=0, atol=1e-11)
    lib = torch.nn.grad.conv2d_weight(torch.from_numpy(x), (J, C, kh, kw), torch.from_numpy(dy),
                                      stride=s, padding=p, dilation=d).numpy()
    np.testing.assert_allclose(got, lib, rtol=0, atol=1e-11)
    np.testing.assert_array_equal(oracle.dw_conv(x, dy, kh, kw, s, p, d, 1, 2), got[1:2])


def test_conv_1x1_equals_fc_on_nhwc_tokens():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 5, 4, 6))
    dy = rng.standard_normal((2, 7, 4, 6))
    conv = oracle.dw_conv(x, dy, 1, 1)[:, :, 0, 0]
    fc = oracle.dw_fc(x.transpose(0, 2, 3, 1), dy.transpose(0, 2, 3, 1))
    np.testing.assert_allclose(conv, fc, rtol=0, atol=1e-12)


@pytest.mark.parametrize("pos", [(0, 0), (0, 5), (5, 0), (5, 5), (2, 3)])
def test_conv_single_retained_element_closed_form(pos):
    # one nonzero a[n,c,h,w] = s  =>  dW[j,c,u,v] = s * dY[n,j,h+1-u,w+1-v] (zero if outside), 3x3/s1/p1
    H = W = 6
    rng = np.random.default_rng(5)
    dy = rng.standard_normal((2, 3, H, W))
    x = np.zeros((2, 4, H, W))
    n, c, (h, w), s = 1, 2, pos, -1.75
    x[n, c, h, w] = s
    got = oracle.dw_conv(x, dy, 3, 3, (1, 1), (1, 1))
    want = np.zeros((3, 4, 3, 3))
    for u in range(3):
        for v in range(3):
            oy, ox = h + 1 - u, w + 1 - v
            if 0 <= oy < H and 0 <= ox < W:
                want[:, c, u, v] = s * dy[n, :, oy, ox]
    np.testing.assert_array_equal(got, want)


def test_conv_integer_exact_and_gamma_zero_and_split():
    rng = np.random.default_rng(8)
    xi = rng.integers(-3, 4, (2, 3, 7, 7)).astype(np.float32)
    dyi = rng.integers(-2, 3, (2, 4, 7, 7)).astype(np.float32)
    xw, dyw = oracle.widen(xi), oracle.widen(dyi)
    dense = oracle.dw_conv(xw, dyw, 3, 3, (1, 1), (1, 1))
    assert np.array_equal(dense, np.round(dense))                    # integers stay integers
    vals, idx = oracle.compress(xi, xi.size)                          # gamma = 0
    assert np.array_equal(oracle.dw_conv(oracle.densify(vals, idx, xi.shape), dyw, 3, 3, (1, 1), (1, 1)), dense)
    k = oracle.keep_count(xi.size, 0.8)
    vals, idx = oracle.compress(xi, k)
    xh = oracle.densify(vals, idx, xi.shape)
    split = oracle.dw_conv(xh, dyw, 3, 3, (1, 1), (1, 1)) + oracle.dw_conv(xw - xh, dyw, 3, 3, (1, 1), (1, 1))
    assert np.array_equal(split, dense)                               # exact: all terms are small integers
