"""Pins for the oracle's non-convolution layers: closed forms, brute force in numpy,
library routines and finite differences on the double build."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _fd_check(f, grad, x, rng, n=16, h=1e-5, tol=1e-6):
    """f: array -> scalar.  Compares central differences at random entries with grad."""
    idx = rng.choice(x.size, size=min(n, x.size), replace=False)
    for i in idx:
        xp, xm = x.copy().ravel(), x.copy().ravel()
        xp[i] += h; xm[i] -= h
        fd = (f(xp.reshape(x.shape)) - f(xm.reshape(x.shape))) / (2 * h)
        assert abs(fd - grad.ravel()[i]) <= tol * max(1.0, abs(fd)), (i, fd, grad.ravel()[i])


def test_relu(orc32):
    x = np.array([-2.0, -0.0, 0.0, 1e-30, 3.5], np.float32)
    assert np.array_equal(orc32.relu_fwd(x), np.array([0, 0, 0, 1e-30, 3.5], np.float32))
    dy = np.arange(1, 6, dtype=np.float32)
    assert np.array_equal(orc32.relu_bwd(x, dy), np.array([0, 0, 0, 4, 5], np.float32))  # ReLU'(0) = 0


@pytest.mark.parametrize("H,k,s,p,expect", [(55, 3, 2, 0, 27), (27, 3, 2, 0, 13), (13, 3, 2, 0, 6),
                                            (28, 3, 1, 1, 28), (8, 3, 2, 0, 4), (6, 2, 2, 1, 4)])
def test_maxpool_output_size(orc32, H, k, s, p, expect):
    assert orc32.maxpool_out(H, k, s, p) == expect


@pytest.mark.parametrize("shape,k,s,p", [((2, 3, 13, 13), 3, 2, 0), ((1, 2, 9, 7), 3, 1, 1), ((1, 1, 8, 8), 3, 2, 0)])
def test_maxpool_vs_library_and_brute_force(orc64, shape, k, s, p):
    rng = np.random.default_rng(5)
    x = rng.standard_normal(shape)
    y, am = orc64.maxpool_fwd(x, k, s, p)
    ref, idx = F.max_pool2d(torch.from_numpy(x), k, s, p, ceil_mode=True, return_indices=True)
    assert np.array_equal(y, ref.numpy())
    assert np.array_equal(am, idx.numpy().astype(np.int32))
    dy = rng.standard_normal(y.shape)
    dx = orc64.maxpool_bwd(shape, k, s, p, dy, am)
    # brute force: scatter each dy to the position its window's maximum came from
    expect = np.zeros(shape)
    N, C, H, W = shape
    for n in range(N):
        for c in range(C):
            for oh in range(y.shape[2]):
                for ow in range(y.shape[3]):
                    win = [(x[n, c, ih, iw], -ih * W - iw, ih, iw)
                           for ih in range(oh * s - p, oh * s - p + k) if 0 <= ih < H
                           for iw in range(ow * s - p, ow * s - p + k) if 0 <= iw < W]
                    _, _, ih, iw = max(win)
                    expect[n, c, ih, iw] += dy[n, c, oh, ow]
    np.testing.assert_allclose(dx, expect, atol=1e-14)


def test_maxpool_ties_take_the_first_maximum(orc32):
    x = np.zeros((1, 1, 4, 4), np.float32)
    y, am = orc32.maxpool_fwd(x, 2, 2, 0)
    assert np.array_equal(am.ravel(), [0, 2, 8, 10])
    x[0, 0, 1, 1] = x[0, 0, 0, 1] = 1.0
    _, am = orc32.maxpool_fwd(x, 2, 2, 0)
    assert am.ravel()[0] == 1


def test_maxpool_padding_never_wins(orc32):
    x = -np.ones((1, 1, 3, 3), np.float32)
    y, _ = orc32.maxpool_fwd(x, 3, 1, 1)
    assert np.array_equal(y, x)


def test_lrn_closed_form_and_library(orc64):
    # constant input v over C channels: interior channels see `size` terms
    C, size, alpha, beta, kappa, v = 9, 5, 1e-2, 0.75, 2.0, 3.0
    x = np.full((1, C, 2, 2), v)
    y, sc = orc64.lrn_fwd(x, size, alpha, beta, kappa)
    cnt = np.array([min(c + 2, C - 1) - max(c - 2, 0) + 1 for c in range(C)])
    np.testing.assert_allclose(sc[0, :, 0, 0], kappa + alpha / size * cnt * v * v, rtol=1e-15)
    np.testing.assert_allclose(y[0, :, 1, 1], v * (kappa + alpha / size * cnt * v * v) ** -beta, rtol=1e-14)
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 7, 3, 4))
    y, _ = orc64.lrn_fwd(x, 5, 1e-1, 0.75, 1.0)
    ref = F.local_response_norm(torch.from_numpy(x), 5, alpha=1e-1, beta=0.75, k=1.0).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12)


@pytest.mark.parametrize("size", [5, 3])
def test_lrn_backward_by_finite_differences(orc64, size):
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 8, 3, 3)) * 2
    alpha, beta, kappa = 0.3, 0.75, 1.0      # large alpha so the cross term matters
    r = rng.standard_normal(x.shape)
    y, sc = orc64.lrn_fwd(x, size, alpha, beta, kappa)
    dx = orc64.lrn_bwd(x, y, sc, r, size, alpha, beta)
    _fd_check(lambda a: float((orc64.lrn_fwd(a, size, alpha, beta, kappa)[0] * r).sum()), dx, x, rng, n=40)


def test_avgpool(orc64):
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 4, 5, 6))
    np.testing.assert_allclose(orc64.avgpool_fwd(x)[:, :, 0, 0], x.mean(axis=(2, 3)), rtol=1e-14)
    assert np.array_equal(orc64.avgpool_fwd(np.full((1, 2, 3, 3), 1.25)), np.full((1, 2, 1, 1), 1.25))
    dy = rng.standard_normal((3, 4, 1, 1))
    dx = orc64.avgpool_bwd(x.shape, dy)
    np.testing.assert_allclose(dx, np.broadcast_to(dy / 30.0, x.shape), rtol=1e-15)


def test_fc_vs_matrix_products(orc64):
    rng = np.random.default_rng(9)
    B, IN, OUT = 5, 7, 4
    x, W, b, dy = rng.standard_normal((B, IN)), rng.standard_normal((OUT, IN)), rng.standard_normal(OUT), \
        rng.standard_normal((B, OUT))
    np.testing.assert_allclose(orc64.fc_fwd(x, W, b), x @ W.T + b, atol=1e-13)
    np.testing.assert_allclose(orc64.fc_bwd_data(dy, W), dy @ W, atol=1e-13)
    dW, db = orc64.fc_bwd_weight(x, dy)
    np.testing.assert_allclose(dW, dy.T @ x, atol=1e-13)
    np.testing.assert_allclose(db, dy.sum(0), atol=1e-13)


def test_dropout(orc32):
    x = np.arange(1, 9, dtype=np.float32)
    mask = np.array([1, 0, 1, 1, 0, 0, 1, 0], np.uint8)
    assert np.array_equal(orc32.dropout(x, mask, 0.5), x * mask * 2)
    np.testing.assert_allclose(orc32.dropout(x, mask, 0.2), x * mask / np.float32(0.8), rtol=1e-7)


def test_softmax_ce_closed_forms(orc64):
    for C in (10, 1000):
        B = 4
        labels = np.array([0, 3, C - 1, 5], np.int32)
        loss, dz = orc64.softmax_ce(np.zeros((B, C)), labels)
        assert abs(loss - math.log(C)) < 1e-14
        expect = np.full((B, C), 1.0 / C)
        expect[np.arange(B), labels] -= 1.0
        np.testing.assert_allclose(dz, expect / B, atol=1e-16)
    # shift invariance and a large-logit case that overflows without max subtraction
    z = np.array([[1000.0, 999.0, 0.0]])
    loss, _ = orc64.softmax_ce(z, np.array([1], np.int32))
    assert abs(loss - (1.0 + math.log1p(math.exp(-1.0)))) < 1e-12


def test_softmax_ce_vs_library_and_fd(orc64):
    rng = np.random.default_rng(10)
    B, C = 6, 11
    z = rng.standard_normal((B, C)) * 3
    labels = rng.integers(0, C, B).astype(np.int32)
    loss, dz = orc64.softmax_ce(z, labels)
    ref = F.cross_entropy(torch.from_numpy(z), torch.from_numpy(labels).long()).item()
    assert abs(loss - ref) < 1e-13
    _fd_check(lambda a: float(orc64.softmax_ce(a, labels)[0]), dz, z, rng, n=30)
