"""Pins for the convolution oracle: nothing here compares the oracle with itself.

Forward is pinned by a hand-worked example, closed forms, an explicit im2col x GEMM
written independently in numpy, and a library routine; the two adjoints are pinned by
finite differences on the double build, by the adjoint identities <conv(x,w),r> =
<x,bwd_data(r,w)> = <w,bwd_weight(x,r)>, and by the stride-1 "flipped kernel" identity.
"""
import os

import numpy as np
import pytest
import torch

from oracle.cgo import conv_desc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "conv_hand_example.txt")

CASES = [
    # N, C, H, W, M, k, stride, pad, groups
    (2, 3, 7, 6, 4, 3, 1, 1, 1),
    (1, 4, 9, 9, 6, 3, 2, 0, 2),
    (2, 2, 11, 10, 3, 5, 1, 2, 1),
    (1, 3, 23, 23, 4, 11, 4, 0, 1),
    (2, 6, 5, 5, 4, 1, 1, 0, 2),
    (1, 2, 8, 8, 2, 3, 3, 2, 1),
]


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _im2col_conv(x, w, b, stride, pad, groups):
    """Independent formulation: explicit column matrix, then one matrix product per group."""
    N, C, H, W = x.shape
    M, Cg, KH, KW = w.shape
    OH, OW = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, M, OH, OW))
    Mg = M // groups
    for n in range(N):
        for g in range(groups):
            col = np.zeros((Cg * KH * KW, OH * OW))
            r = 0
            for c in range(Cg):
                for kh in range(KH):
                    for kw in range(KW):
                        patch = xp[n, g * Cg + c, kh:kh + stride * OH:stride, kw:kw + stride * OW:stride]
                        col[r] = patch.reshape(-1)
                        r += 1
            wm = w[g * Mg:(g + 1) * Mg].reshape(Mg, -1)
            y[n, g * Mg:(g + 1) * Mg] = (wm @ col).reshape(Mg, OH, OW)
    return y + (b.reshape(1, M, 1, 1) if b is not None else 0.0)


def _read_gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = np.array([float(t) for t in v])
    return out


def test_hand_worked_example(orc32, orc64):
    g = _read_gold()
    for orc in (orc32, orc64):
        x = g["x"].reshape(1, 1, 3, 3)
        w = g["w"].reshape(1, 1, 2, 2)
        d = conv_desc(1, 1, 3, 3, 1, 2)
        assert np.array_equal(orc.conv_fwd(d, x, w, g["b"]).ravel(), g["y"])
        d2 = conv_desc(1, 1, 3, 3, 1, 2, stride=2, pad=1)
        assert np.array_equal(orc.conv_fwd(d2, x, w, g["b"]).ravel(), g["y_p1s2"])
        ones = np.ones((1, 1, 2, 2))
        assert np.array_equal(orc.conv_bwd_data(d, ones, w).ravel(), g["dx_ones"])
        dw, db = orc.conv_bwd_weight(d, x, ones)
        assert np.array_equal(dw.ravel(), g["dw_ones"]) and db[0] == 4.0


@pytest.mark.parametrize("case", CASES)
def test_fwd_vs_im2col_gemm(orc64, case):
    N, C, H, W, M, k, s, p, G = case
    rng = np.random.default_rng(11)
    x, w, b = _rand(rng, N, C, H, W), _rand(rng, M, C // G, k, k), _rand(rng, M)
    y = orc64.conv_fwd(conv_desc(N, C, H, W, M, k, s, p, G), x, w, b)
    ref = _im2col_conv(x, w, b, s, p, G)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_fwd_vs_library_routine(orc32, case):
    N, C, H, W, M, k, s, p, G = case
    rng = np.random.default_rng(12)
    x, w, b = (a.astype(np.float32) for a in (_rand(rng, N, C, H, W), _rand(rng, M, C // G, k, k), _rand(rng, M)))
    y = orc32.conv_fwd(conv_desc(N, C, H, W, M, k, s, p, G), x, w, b)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=s, padding=p, groups=G).numpy()
    np.testing.assert_allclose(y, ref, rtol=0, atol=2e-6 * np.abs(ref).max())


def test_rectangular_kernel_and_image(orc64):
    """KH != KW and H != W: catches swapped height/width indices."""
    rng = np.random.default_rng(13)
    x, w = _rand(rng, 2, 2, 6, 9), _rand(rng, 3, 2, 2, 4)
    d = conv_desc(2, 2, 6, 9, 3, 2, stride=1, pad=1, kw=4)
    y = orc64.conv_fwd(d, x, w, None)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), None, stride=1, padding=1).numpy()
    np.testing.assert_allclose(y, ref, atol=1e-12)


def test_delta_kernel_is_shifted_strided_copy(orc32):
    rng = np.random.default_rng(1)
    N, C, H, W, k, s, p = 2, 3, 10, 9, 3, 2, 1
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    for (c0, kh0, kw0) in [(0, 0, 0), (2, 1, 2), (1, 2, 0)]:
        w = np.zeros((1, C, k, k), np.float32)
        w[0, c0, kh0, kw0] = 1.0
        y = orc32.conv_fwd(conv_desc(N, C, H, W, 1, k, s, p), x, w, None)
        xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
        OH, OW = y.shape[2:]
        expect = xp[:, c0, kh0:kh0 + s * OH:s, kw0:kw0 + s * OW:s]
        assert np.array_equal(y[:, 0], expect)


def test_all_ones_counts_in_bounds_taps(orc32):
    N, C, H, W, M, k, s, p, G = 1, 4, 6, 7, 2, 3, 1, 1, 2
    y = orc32.conv_fwd(conv_desc(N, C, H, W, M, k, s, p, G), np.ones((N, C, H, W)), np.ones((M, C // G, k, k)), None)
    rows = np.array([min(i + 1, H - 1) - max(i - 1, 0) + 1 for i in range(H)])
    cols = np.array([min(j + 1, W - 1) - max(j - 1, 0) + 1 for j in range(W)])
    expect = (C // G) * np.outer(rows, cols)
    assert np.array_equal(y[0, 0], expect) and np.array_equal(y[0, 1], expect)


def test_one_by_one_is_per_pixel_matrix_product(orc64):
    rng = np.random.default_rng(2)
    x, w = _rand(rng, 2, 5, 4, 3), _rand(rng, 7, 5, 1, 1)
    y = orc64.conv_fwd(conv_desc(2, 5, 4, 3, 7, 1), x, w, None)
    np.testing.assert_allclose(y, np.einsum("mc,nchw->nmhw", w[:, :, 0, 0], x), atol=1e-13)


def test_groups_are_independent_convolutions(orc64):
    rng = np.random.default_rng(3)
    N, C, H, M, k, G = 2, 6, 7, 4, 3, 2
    x, w, b = _rand(rng, N, C, H, H), _rand(rng, M, C // G, k, k), _rand(rng, M)
    y = orc64.conv_fwd(conv_desc(N, C, H, H, M, k, 1, 1, G), x, w, b)
    for g in range(G):
        xs = x[:, g * 3:(g + 1) * 3]
        ys = orc64.conv_fwd(conv_desc(N, 3, H, H, 2, k, 1, 1, 1), xs, w[g * 2:(g + 1) * 2], b[g * 2:(g + 1) * 2])
        np.testing.assert_allclose(y[:, g * 2:(g + 1) * 2], ys, atol=1e-13)
    # the second group's input must not leak into the first group's output
    x2 = x.copy(); x2[:, 3:] += 1.0
    y2 = orc64.conv_fwd(conv_desc(N, C, H, H, M, k, 1, 1, G), x2, w, b)
    assert np.array_equal(y2[:, :2], y[:, :2]) and not np.array_equal(y2[:, 2:], y[:, 2:])


@pytest.mark.parametrize("case", CASES)
def test_backward_by_finite_differences(orc64, case):
    """conv is bilinear, so central differences of L = <y, r> are exact up to rounding."""
    N, C, H, W, M, k, s, p, G = case
    rng = np.random.default_rng(21)
    d = conv_desc(N, C, H, W, M, k, s, p, G)
    x, w, b = _rand(rng, N, C, H, W), _rand(rng, M, C // G, k, k), _rand(rng, M)
    r = _rand(rng, *orc64.conv_fwd(d, x, w, b).shape)
    dx = orc64.conv_bwd_data(d, r, w)
    dw, db = orc64.conv_bwd_weight(d, x, r)

    def L(x_, w_, b_):
        return float((orc64.conv_fwd(d, x_, w_, b_) * r).sum())

    h = 1e-3
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        idx = rng.choice(arr.size, size=min(12, arr.size), replace=False)
        for i in idx:
            ap, am = arr.copy().ravel(), arr.copy().ravel()
            ap[i] += h; am[i] -= h
            args_p = [x, w, b]; args_m = [x, w, b]
            args_p[which] = ap.reshape(arr.shape); args_m[which] = am.reshape(arr.shape)
            fd = (L(*args_p) - L(*args_m)) / (2 * h)
            assert abs(fd - grad.ravel()[i]) <= 1e-8 * max(1.0, abs(fd)), (which, i)


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities(orc64, case):
    N, C, H, W, M, k, s, p, G = case
    rng = np.random.default_rng(22)
    d = conv_desc(N, C, H, W, M, k, s, p, G)
    x, w = _rand(rng, N, C, H, W), _rand(rng, M, C // G, k, k)
    y = orc64.conv_fwd(d, x, w, None)
    r = _rand(rng, *y.shape)
    lhs = (y * r).sum()
    dw, db = orc64.conv_bwd_weight(d, x, r)
    assert abs(lhs - (x * orc64.conv_bwd_data(d, r, w)).sum()) <= 1e-10 * abs(lhs) + 1e-10
    assert abs(lhs - (w * dw).sum()) <= 1e-10 * abs(lhs) + 1e-10
    np.testing.assert_allclose(db, r.sum(axis=(0, 2, 3)), atol=1e-12)


def test_stride1_bwd_data_is_conv_with_flipped_transposed_kernel(orc64):
    rng = np.random.default_rng(23)
    N, C, H, W, M, k, p = 2, 3, 8, 7, 5, 3, 1
    w, dy = _rand(rng, M, C, k, k), _rand(rng, N, M, H, W)
    dx = orc64.conv_bwd_data(conv_desc(N, C, H, W, M, k, 1, p), dy, w)
    wt = np.ascontiguousarray(w.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    ref = torch.nn.functional.conv2d(torch.from_numpy(dy), torch.from_numpy(wt), None, padding=k - 1 - p).numpy()
    np.testing.assert_allclose(dx, ref, atol=1e-12)


def test_float_build_rounds_the_double_result_once(orc32, orc64):
    rng = np.random.default_rng(24)
    N, C, H, W, M, k, s, p, G = CASES[0]
    d = conv_desc(N, C, H, W, M, k, s, p, G)
    x, w, b = (a.astype(np.float32) for a in (_rand(rng, N, C, H, W), _rand(rng, M, C // G, k, k), _rand(rng, M)))
    y32 = orc32.conv_fwd(d, x, w, b)
    y64 = orc64.conv_fwd(d, x, w, b)
    assert y32.dtype == np.float32 and np.array_equal(y32, y64.astype(np.float32))


def test_bad_descriptor_is_rejected(orc32):
    with pytest.raises(ValueError):
        orc32.conv_out_shape(conv_desc(1, 3, 4, 4, 4, 5))       # kernel larger than image
    with pytest.raises(ValueError):
        orc32.conv_out_shape(conv_desc(1, 3, 8, 8, 4, 3, groups=2))  # C not divisible
