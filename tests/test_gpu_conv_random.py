"""Randomised differential test of the three convolution passes: 48 seeded descriptors with
independent kernel heights and widths, strides and paddings per axis, groups and ragged sizes, each
run through the default kernel choice and again with the thresholds lowered that normally keep
the raw-row (patch) kernels and the two-launch forward for large problems.  Reference: the CPU
oracle's direct loops; tolerance as everywhere, max-abs-relative <= 1e-3."""
import numpy as np
import pytest
import torch

import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_data, conv_bwd_weight, conv_fwd, dev, host, max_abs_rel
from oracle.cgo import ConvDesc

pytestmark = pytest.mark.gpu
TOL = 1e-3
N_CASES = 48


def _case(i):
    rng = np.random.default_rng(1000 + i)
    groups = int(rng.choice([1, 1, 1, 2, 3, 4]))
    Cg = int(rng.choice([1, 2, 3, 5, 8, 16, 16, 32, 48]))
    Mg = int(rng.choice([1, 4, 7, 16, 24, 33, 48, 64, 100]))
    KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    if rng.random() < 0.3:
        KW = KH
    sh = int(rng.choice([1, 1, 1, 2, 3]))
    sw = sh if rng.random() < 0.6 else int(rng.choice([1, 2, 3]))
    ph, pw = int(rng.integers(0, KH)), int(rng.integers(0, KW))
    H = int(rng.integers(max(KH - 2 * ph, 1), 26))
    W = int(rng.integers(max(KW - 2 * pw, 1), 26))
    B = int(rng.integers(1, 5))
    return dict(N=B, C=Cg * groups, H=H, W=W, M=Mg * groups, KH=KH, KW=KW, sh=sh, sw=sw, ph=ph, pw=pw, groups=groups)


def _tensors(c, seed):
    rng = np.random.default_rng(seed)
    Cg, Mg = c["C"] // c["groups"], c["M"] // c["groups"]
    OH = (c["H"] + 2 * c["ph"] - c["KH"]) // c["sh"] + 1
    OW = (c["W"] + 2 * c["pw"] - c["KW"]) // c["sw"] + 1
    fi, fo = Cg * c["KH"] * c["KW"], Mg * c["KH"] * c["KW"]
    x = rng.standard_normal((c["N"], c["C"], c["H"], c["W"]), dtype=np.float32) / np.float32(np.sqrt(fi))
    w = rng.standard_normal((c["M"], Cg, c["KH"], c["KW"]), dtype=np.float32) / np.float32(np.sqrt(fi))
    b = rng.standard_normal(c["M"], dtype=np.float32) * np.float32(0.1)
    dy = rng.standard_normal((c["N"], c["M"], OH, OW), dtype=np.float32) / np.float32(np.sqrt(fo))
    return x, w, b, dy


@pytest.fixture(params=["default", "low_thresholds"])
def thresholds(request):
    if request.param == "low_thresholds":
        cg.cg_debug_patch_min_tiles(1)
        cg.cg_debug_resident_blocks(3)
    yield request.param
    cg.cg_debug_patch_min_tiles(512)
    cg.cg_debug_resident_blocks(512)


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_descriptor(orc32, thresholds, i):
    c = _case(i)
    args = (c["N"], c["C"], c["H"], c["W"], c["M"], c["KH"], c["KW"], c["sh"], c["sw"], c["ph"], c["pw"], c["groups"])
    d, od = cg.cg_conv_desc(*args), ConvDesc(*args)
    x, w, b, dy = _tensors(c, 5000 + i)
    ry = orc32.conv_fwd(od, x, w, b)
    gy = host(conv_fwd(d, dev(x), dev(w), dev(b)))
    assert gy.shape == ry.shape and np.isfinite(gy).all(), c
    assert max_abs_rel(gy, ry) <= TOL, ("forward", c)
    rdx = orc32.conv_bwd_data(od, dy, w)
    gdx = host(conv_bwd_data(d, dev(dy), dev(w)))
    assert np.isfinite(gdx).all() and max_abs_rel(gdx, rdx) <= TOL, ("backward-data", c)
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    gdw, gdb = conv_bwd_weight(d, dev(x), dev(dy))
    assert max_abs_rel(host(gdw), rdw) <= TOL, ("backward-weight", c)
    assert max_abs_rel(host(gdb), rdb) <= TOL, ("bias gradient", c)


def _medium_case(i):
    """At least 70 000 output pixels: enough tiles for the kernels that stage raw image rows to be the
    default choice, on image sizes whose 128-pixel tiles start and end anywhere."""
    rng = np.random.default_rng(31000 + i)
    g = int(rng.choice([1, 1, 2]))
    Cg = int(rng.choice([16, 16, 32, 48, 64]))
    Mg = int(rng.choice([16, 32, 48, 64, 96, 128, 200]))
    K = int(rng.choice([3, 3, 5]))
    s = int(rng.choice([1, 1, 1, 2]))
    p = int(rng.integers(0, K // 2 + 1))
    H, W = int(rng.integers(7, 34)), int(rng.integers(7, 34))
    OH, OW = (H + 2 * p - K) // s + 1, (W + 2 * p - K) // s + 1
    B = int(np.ceil(70000 / (OH * OW))) + int(rng.integers(0, 7))
    return dict(N=B, C=Cg * g, H=H, W=W, M=Mg * g, KH=K, KW=K, sh=s, sw=s, ph=p, pw=p, groups=g)


@pytest.mark.parametrize("i", range(10))
def test_random_medium_descriptor(orc32, i):
    c = _medium_case(i)
    args = (c["N"], c["C"], c["H"], c["W"], c["M"], c["KH"], c["KW"], c["sh"], c["sw"], c["ph"], c["pw"], c["groups"])
    d, od = cg.cg_conv_desc(*args), ConvDesc(*args)
    x, w, b, dy = _tensors(c, 41000 + i)
    assert max_abs_rel(host(conv_fwd(d, dev(x), dev(w), dev(b))), orc32.conv_fwd(od, x, w, b)) <= TOL, ("forward", c)
    assert max_abs_rel(host(conv_bwd_data(d, dev(dy), dev(w))), orc32.conv_bwd_data(od, dy, w)) <= TOL, ("backward-data", c)
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    gdw, gdb = conv_bwd_weight(d, dev(x), dev(dy))
    assert max_abs_rel(host(gdw), rdw) <= TOL, ("backward-weight", c)
    assert max_abs_rel(host(gdb), rdb) <= TOL, ("bias gradient", c)
