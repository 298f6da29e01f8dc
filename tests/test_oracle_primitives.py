"""Pins for the oracle's primitives against things other than the oracle itself:
brute force, closed forms, special cases that reduce to a matrix product,
adjoint identities and PyTorch's CPU fp64 library routines."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pbd_oracle as orc

RNG = np.random.default_rng(1234)
CONV_CASES = [  # N, C, H, W, K, k, stride, groups
    (2, 3, 7, 6, 4, 3, 1, 1), (2, 4, 8, 8, 6, 3, 2, 1), (1, 5, 6, 7, 3, 1, 1, 1),
    (2, 4, 9, 9, 4, 5, 2, 4), (1, 3, 11, 10, 3, 7, 1, 3), (2, 6, 8, 8, 6, 3, 2, 6),
    (1, 3, 12, 12, 5, 7, 2, 1), (2, 8, 5, 5, 4, 1, 2, 1),
]


def brute_conv(x, w, stride, pad, groups):
    """Textbook cross-correlation written as a scatter over input pixels."""
    N, C, H, W = x.shape
    K, Cg, k, _ = w.shape
    P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.zeros((N, K, P, Q))
    Kg = K // groups
    for n, c, h, ww in itertools.product(range(N), range(C), range(H), range(W)):
        g = c // Cg
        for r, t in itertools.product(range(k), range(k)):
            ph, qw = h + pad - r, ww + pad - t
            if ph % stride or qw % stride:
                continue
            p, q = ph // stride, qw // stride
            if 0 <= p < P and 0 <= q < Q:
                y[n, g * Kg:(g + 1) * Kg, p, q] += x[n, c, h, ww] * w[g * Kg:(g + 1) * Kg, c - g * Cg, r, t]
    return y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_brute_force_and_library(case):
    N, C, H, W, K, k, s, g = case
    x = RNG.standard_normal((N, C, H, W))
    w = RNG.standard_normal((K, C // g, k, k))
    y = orc.conv_fwd(x, w, s, k // 2, g)
    np.testing.assert_allclose(y, brute_conv(x, w, s, k // 2, g), rtol=0, atol=1e-12)
    yt = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=s, padding=k // 2, groups=g)
    np.testing.assert_allclose(y, yt.numpy(), rtol=0, atol=1e-12)


def test_conv_1x1_is_matrix_product():
    x = RNG.standard_normal((3, 5, 4, 6))
    w = RNG.standard_normal((7, 5, 1, 1))
    y = orc.conv_fwd(x, w)
    np.testing.assert_allclose(y, np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x), atol=1e-13)


def test_conv_on_single_pixel_is_centre_tap():
    x = RNG.standard_normal((4, 6, 1, 1))
    w = RNG.standard_normal((5, 6, 3, 3))
    y = orc.conv_fwd(x, w, 1, 1)
    np.testing.assert_allclose(y[:, :, 0, 0], x[:, :, 0, 0] @ w[:, :, 1, 1].T, atol=1e-13)


def test_conv_delta_kernel_shifts():
    x = RNG.standard_normal((1, 1, 6, 6))
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 2] = 1.0      # tap at r=0, t=2: y[p,q] = x[p-1, q+1]
    y = orc.conv_fwd(x, w, 1, 1)
    ref = np.zeros_like(x)
    ref[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y, ref)


def test_depthwise_is_block_diagonal_dense():
    C = 5
    x = RNG.standard_normal((2, C, 7, 7))
    w = RNG.standard_normal((C, 1, 3, 3))
    wd = np.zeros((C, C, 3, 3))
    for c in range(C):
        wd[c, c] = w[c, 0]
    np.testing.assert_allclose(orc.conv_fwd(x, w, 2, 1, C), orc.conv_fwd(x, wd, 2, 1, 1), atol=1e-13)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_adjoints_and_autograd(case):
    N, C, H, W, K, k, s, g = case
    pad = k // 2
    x = RNG.standard_normal((N, C, H, W))
    w = RNG.standard_normal((K, C // g, k, k))
    y = orc.conv_fwd(x, w, s, pad, g)
    dy = RNG.standard_normal(y.shape)
    dx = orc.conv_dgrad(dy, w, x.shape, s, pad, g)
    dw = orc.conv_wgrad(dy, x, k, s, pad, g)
    lhs = np.sum(y * dy)
    assert abs(lhs - np.sum(x * dx)) <= 1e-11 * max(1.0, abs(lhs))
    assert abs(lhs - np.sum(w * dw)) <= 1e-11 * max(1.0, abs(lhs))
    xt = torch.from_numpy(x).requires_grad_()
    wt = torch.from_numpy(w).requires_grad_()
    F.conv2d(xt, wt, stride=s, padding=pad, groups=g).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.numpy(), atol=1e-11)


def test_bn_train_closed_forms():
    x = RNG.standard_normal((4, 3, 5, 5)) * 2.0 + 1.0
    gamma, beta = RNG.uniform(0.5, 1.5, 3), RNG.standard_normal(3)
    y, mean, var = orc.bn_train_fwd(x, gamma, beta)
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), atol=1e-13)
    np.testing.assert_allclose(var, x.var(axis=(0, 2, 3)), atol=1e-13)       # biased
    xh = (x - mean[None, :, None, None]) / np.sqrt(var + 1e-5)[None, :, None, None]
    np.testing.assert_allclose(y, gamma[None, :, None, None] * xh + beta[None, :, None, None], atol=1e-12)
    # positive rescaling of the input leaves the output unchanged as eps -> 0
    y0, _, _ = orc.bn_train_fwd(x, gamma, beta, eps=0.0)
    y1, _, _ = orc.bn_train_fwd(3.7 * x, gamma, beta, eps=0.0)
    np.testing.assert_allclose(y0, y1, atol=1e-12)
    dy = RNG.standard_normal(x.shape)
    dx, dg, db = orc.bn_train_bwd(dy, x, gamma, mean, var)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), atol=1e-12)
    np.testing.assert_allclose(dg, (dy * xh).sum(axis=(0, 2, 3)), atol=1e-12)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)          # orthogonal to 1
    np.testing.assert_allclose((dx * xh).sum(axis=(0, 2, 3)), 0, atol=1e-4)    # and to xhat (eps)
    xt = torch.from_numpy(x).requires_grad_()
    gt = torch.from_numpy(gamma).requires_grad_()
    bt = torch.from_numpy(beta).requires_grad_()
    F.batch_norm(xt, None, None, gt, bt, training=True, eps=1e-5).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_bn_eval_is_affine():
    x = RNG.standard_normal((2, 4, 3, 3))
    g, b, rm, rv = RNG.uniform(0.5, 1.5, 4), RNG.standard_normal(4), RNG.standard_normal(4), RNG.uniform(0.5, 2, 4)
    y = orc.bn_eval(x, g, b, rm, rv)
    a = g / np.sqrt(rv + 1e-5)
    np.testing.assert_allclose(y, a[None, :, None, None] * x + (b - a * rm)[None, :, None, None], atol=1e-13)


def test_activations():
    x = np.array([-1.0, 0.0, 0.5, 5.9, 6.0, 7.5])
    np.testing.assert_array_equal(orc.act_fwd(x, 0), x)
    np.testing.assert_array_equal(orc.act_fwd(x, 1), [0, 0, 0.5, 5.9, 6.0, 7.5])
    np.testing.assert_array_equal(orc.act_fwd(x, 2), [0, 0, 0.5, 5.9, 6.0, 6.0])
    dy = np.arange(1.0, 7.0)
    np.testing.assert_array_equal(orc.act_bwd(dy, x, 0), dy)
    np.testing.assert_array_equal(orc.act_bwd(dy, x, 1), [0, 0, 3, 4, 5, 6])
    np.testing.assert_array_equal(orc.act_bwd(dy, x, 2), [0, 0, 3, 4, 0, 0])


@pytest.mark.parametrize("k,s,p,H", [(2, 2, 0, 8), (3, 2, 1, 9), (3, 2, 1, 8), (2, 2, 0, 1 + 1)])
def test_maxpool_against_library(k, s, p, H):
    x = RNG.standard_normal((2, 3, H, H + 1))
    y, idx = orc.maxpool_fwd(x, k, s, p)
    xt = torch.from_numpy(x).requires_grad_()
    yt = F.max_pool2d(xt, k, s, p)
    np.testing.assert_array_equal(y, yt.detach().numpy())
    dy = RNG.standard_normal(y.shape)
    yt.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(orc.maxpool_bwd(dy, idx, x.shape), xt.grad.numpy(), atol=1e-14)


def test_maxpool_ties_go_to_first_in_window_order():
    x = np.zeros((1, 1, 2, 4))
    x[0, 0, :, 2:] = [[1.0, 3.0], [3.0, 2.0]]
    y, idx = orc.maxpool_fwd(x, 2, 2, 0)
    np.testing.assert_array_equal(y[0, 0], [[0.0, 3.0]])
    np.testing.assert_array_equal(idx[0, 0], [[0, 3]])        # flat h*W+w of the first maximum
    dx = orc.maxpool_bwd(np.array([[[[5.0, 7.0]]]]), idx, x.shape)
    ref = np.zeros_like(x); ref[0, 0, 0, 0] = 5.0; ref[0, 0, 0, 3] = 7.0
    np.testing.assert_array_equal(dx, ref)


def test_mse_identities():
    s, t = RNG.standard_normal(37), RNG.standard_normal(37)
    loss, ds = orc.mse(s, t)
    assert abs(loss - np.mean((s - t) ** 2)) < 1e-14
    assert abs(np.sum(ds * (s - t)) - 2 * loss) < 1e-13
    loss0, ds0 = orc.mse(s, s)
    assert loss0 == 0.0 and not ds0.any()
    # worked example: s = (1, 2, 4), t = (0, 2, 1): loss = (1 + 0 + 9)/3
    loss1, ds1 = orc.mse(np.array([1.0, 2, 4]), np.array([0.0, 2, 1]))
    assert abs(loss1 - 10.0 / 3.0) < 1e-15
    np.testing.assert_allclose(ds1, [2 / 3, 0, 2.0], atol=1e-15)


def test_sgd_momentum_closed_form():
    g = RNG.standard_normal(5)
    w0 = RNG.standard_normal(5)
    lr, mu = 0.1, 0.9
    w, v = w0.copy(), np.zeros(5)
    vsum = np.zeros(5)
    for kstep in range(1, 6):
        w, v = orc.sgd(w, v, g, lr, mu)
        vk = g * (1 - mu ** kstep) / (1 - mu)
        vsum += vk
        np.testing.assert_allclose(v, vk, atol=1e-13)
        np.testing.assert_allclose(w, w0 - lr * vsum, atol=1e-13)
    w1, v1 = orc.sgd(w0, np.zeros(5), g, lr, 0.0)             # mu = 0 is plain SGD
    np.testing.assert_allclose(w1, w0 - lr * g, atol=1e-15)
