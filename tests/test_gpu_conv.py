"""GPU parity of the three convolution passes against the CPU oracle (direct 7-loop
definition in double, rounded once), element by element; tolerance: max-abs-relative
error <= 1e-3 (fp32 path)."""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_data, conv_bwd_weight, conv_fwd, dev, host, max_abs_rel
from oracle.cgo import conv_desc as odesc

pytestmark = pytest.mark.gpu
TOL = 1e-3

# name -> (B, cfg).  Shapes chosen to hit every tile configuration (M per group 16..384),
# ragged M / N / K tails, K not divisible by 4, groups, strides and paddings, and to span
# several 128-pixel tiles while the oracle still finishes in seconds.
SHAPES = {
    "conv1_like_s4": (3, dict(C=3, H=51, M=96, k=11, stride=4, pad=0, groups=1)),
    "conv2_like_g2": (2, dict(C=16, H=27, M=256, k=5, stride=1, pad=2, groups=2)),
    "conv3_like": (2, dict(C=32, H=13, M=384, k=3, stride=1, pad=1, groups=1)),
    "conv4_like_g2": (3, dict(C=24, H=13, M=384, k=3, stride=1, pad=1, groups=2)),
    "one_by_one_m64": (2, dict(C=20, H=14, M=64, k=1, stride=1, pad=0, groups=1)),
    "tiny_m16": (2, dict(C=6, H=9, M=16, k=1, stride=1, pad=0, groups=1)),
    "five_m32_p2": (2, dict(C=16, H=12, M=32, k=5, stride=1, pad=2, groups=1)),
    "ragged_m100_k3": (1, dict(C=5, H=17, W=11, M=100, k=3, stride=1, pad=1, groups=1)),
    "stride2_pad1": (2, dict(C=8, H=15, M=48, k=3, stride=2, pad=1, groups=1)),
    "stride3_g4": (2, dict(C=8, H=16, M=8, k=4, stride=3, pad=2, groups=4)),
    "cfg1_layer1": (8, dict(C=3, H=32, M=16, k=3, stride=1, pad=1, groups=1)),
    "cfg1_layer2": (8, dict(C=16, H=32, M=32, k=3, stride=1, pad=1, groups=1)),
    "single_pixel": (1, dict(C=4, H=3, M=4, k=3, stride=1, pad=0, groups=1)),
    "seven_s2_g2_nopad": (2, dict(C=8, H=21, W=19, M=24, k=7, stride=2, pad=0, groups=2)),
}


def _setup(name):
    B, cfg = SHAPES[name]
    c, x, w, b, dy = cg_synth.conv_layer_tensors(name, B, seed=sum(map(ord, name)), cfg=cfg)
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], Wd, c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    return d, od, x, w, b, dy


@pytest.mark.parametrize("name", list(SHAPES))
def test_forward(orc32, name):
    d, od, x, w, b, _ = _setup(name)
    ref = orc32.conv_fwd(od, x, w, b)
    got = host(conv_fwd(d, dev(x), dev(w), dev(b)))
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert max_abs_rel(got, ref) <= TOL
    ref0 = orc32.conv_fwd(od, x, w, None)
    assert max_abs_rel(host(conv_fwd(d, dev(x), dev(w), None)), ref0) <= TOL


@pytest.mark.parametrize("name", list(SHAPES))
def test_backward_data(orc32, name):
    d, od, x, w, b, dy = _setup(name)
    ref = orc32.conv_bwd_data(od, dy, w)
    got = host(conv_bwd_data(d, dev(dy), dev(w)))
    assert np.isfinite(got).all()
    assert max_abs_rel(got, ref) <= TOL


@pytest.mark.parametrize("name", list(SHAPES))
def test_backward_weight(orc32, name):
    d, od, x, w, b, dy = _setup(name)
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    gdw, gdb = conv_bwd_weight(d, dev(x), dev(dy))
    gdw, gdb = host(gdw), host(gdb)
    assert np.isfinite(gdw).all() and np.isfinite(gdb).all()
    assert max_abs_rel(gdw, rdw) <= TOL
    assert max_abs_rel(gdb, rdb) <= TOL


def test_backward_weight_is_reproducible_and_bias_optional():
    d, od, x, w, b, dy = _setup("conv3_like")
    dx_, dy_ = dev(x), dev(dy)
    a, _ = conv_bwd_weight(d, dx_, dy_)
    b2, _ = conv_bwd_weight(d, dx_, dy_)
    assert torch.equal(a, b2)
    dw = torch.empty_like(a)
    ws = torch.empty(max(cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT), 16), dtype=torch.uint8, device="cuda")
    cg.cg_conv_bwd_weight(d, dx_, dy_, dw, None, ws)
    assert torch.equal(dw, a)


def test_workspace_too_small_is_an_error():
    d, od, x, w, b, dy = _setup("conv3_like")
    dx = torch.empty((d.N, d.C, d.H, d.W), device="cuda")
    with pytest.raises(cg.CgError) as e:
        cg.cg_conv_bwd_data(d, dev(dy), dev(w), dx, torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == cg.CG_ENOSPC


@pytest.mark.parametrize("layer", ["conv2", "conv3", "conv5"])
def test_alexnet_layer_small_batch_full_spatial_size(orc32, layer):
    """The real layer geometry (channels, image, filter, groups) at B=4."""
    B = 4
    c, x, w, b, dy = cg_synth.conv_layer_tensors(layer, B, seed=2)
    d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], c["H"], c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    dx_, dw_, db_, dy_ = dev(x), dev(w), dev(b), dev(dy)
    assert max_abs_rel(host(conv_fwd(d, dx_, dw_, db_)), orc32.conv_fwd(od, x, w, b)) <= TOL
    assert max_abs_rel(host(conv_bwd_data(d, dy_, dw_)), orc32.conv_bwd_data(od, dy, w)) <= TOL
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    gdw, gdb = conv_bwd_weight(d, dx_, dy_)
    assert max_abs_rel(host(gdw), rdw) <= TOL and max_abs_rel(host(gdb), rdb) <= TOL


# Shapes that qualify for the patch kernel (reduction channels per group a multiple of 16, at least
# five taps) once the tile threshold is lowered: padded borders, 5x5 windows, stride 2, groups, row
# tiles of 64 / 128 / 192, pixel tiles that span two and more images, ragged last tiles, and images
# large enough that blocks are confined to one image (27x27 with a 5x5 window).
PATCH_SHAPES = {
    "p3x3_13_c32_m128": (3, dict(C=32, H=13, M=128, k=3, stride=1, pad=1, groups=1)),
    "p3x3_13_g2_m384": (2, dict(C=32, H=13, M=384, k=3, stride=1, pad=1, groups=2)),
    "p5x5_27_g2": (1, dict(C=32, H=27, M=64, k=5, stride=1, pad=2, groups=2)),
    "p3x3_7_many_images": (9, dict(C=16, H=7, M=48, k=3, stride=1, pad=1, groups=1)),
    "p3x3_s2_p1": (2, dict(C=16, H=15, M=32, k=3, stride=2, pad=1, groups=1)),
    "p3x3_nopad_w11": (2, dict(C=16, H=17, W=11, M=100, k=3, stride=1, pad=0, groups=1)),
    "p2x3_like_5taps": (2, dict(C=16, H=9, M=16, k=3, stride=1, pad=2, groups=1)),
}


@pytest.fixture
def patch_path():
    cg.cg_debug_patch_min_tiles(1)
    yield
    cg.cg_debug_patch_min_tiles(512)


def _setup_patch(name):
    B, cfg = PATCH_SHAPES[name]
    c, x, w, b, dy = cg_synth.conv_layer_tensors(name, B, seed=sum(map(ord, name)), cfg=cfg)
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], Wd, c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    return d, od, x, w, b, dy


@pytest.mark.parametrize("name", list(PATCH_SHAPES))
def test_patch_kernel_forward(orc32, patch_path, name):
    d, od, x, w, b, dy = _setup_patch(name)
    assert cg.cg_conv_workspace_bytes(d, cg.CG_PASS_FWD) >= w.size * 4        # the tap-major filter copy: patch path taken
    ref = orc32.conv_fwd(od, x, w, b)
    got = host(conv_fwd(d, dev(x), dev(w), dev(b)))
    assert got.shape == ref.shape and np.isfinite(got).all()
    assert max_abs_rel(got, ref) <= TOL


@pytest.mark.parametrize("name", [n for n, (_, c) in PATCH_SHAPES.items() if c["stride"] == 1])
def test_patch_kernel_backward_data(orc32, patch_path, name):
    d, od, x, w, b, dy = _setup_patch(name)
    ref = orc32.conv_bwd_data(od, dy, w)
    got = host(conv_bwd_data(d, dev(dy), dev(w)))
    assert np.isfinite(got).all()
    assert max_abs_rel(got, ref) <= TOL


# A launch whose last round of resident blocks would be mostly empty goes out as two launches:
# the pixel tiles of the whole rounds with the large row tile, the rest with 64-row tiles.  With
# the resident-block count lowered, these shapes take that path (B images of 13x13 pixels).
@pytest.mark.parametrize("B,M,groups,resident", [(3, 128, 1, 3), (5, 384, 2, 12), (7, 256, 1, 6)])
def test_patch_kernel_two_launches(orc32, patch_path, B, M, groups, resident):
    cfg = dict(C=32, H=13, M=M, k=3, stride=1, pad=1, groups=groups)
    c, x, w, b, dy = cg_synth.conv_layer_tensors("two_launch", B, seed=B * 1000 + M, cfg=cfg)
    d = cg.conv_desc(B, c["C"], 13, 13, M, 3, stride=1, pad=1, groups=groups)
    od = odesc(B, c["C"], 13, 13, M, 3, 1, 1, groups)
    ref = orc32.conv_fwd(od, x, w, b)
    cg.cg_debug_resident_blocks(resident)
    cg.cg_profile_enable(True)
    try:
        got = host(conv_fwd(d, dev(x), dev(w), dev(b)))
        names = [cg.cg_profile_get(i)["kernel"] for i in range(cg.cg_profile_count())]
    finally:
        cg.cg_profile_enable(False)
        cg.cg_debug_resident_blocks(512)
    assert len([n for n in names if n.startswith("igemm_patch_kernel")]) == 2, names
    assert max_abs_rel(got, ref) <= TOL


@pytest.mark.parametrize("B,C,M,W", [(2, 16, 64, 56), (1, 64, 160, 56), (2, 32, 128, 52)])
def test_patch_kernel_six_chunks(orc32, patch_path, B, C, M, W):
    """Planes 56 (52) wide with a 3x3 window: the 128 pixels of a block span four pixel rows, 348 (324)
    patch slots a channel, which take the six-chunk instances (64- and 128-row tiles) in forward and,
    where the group has more than 48 input channels, in backward-data."""
    cfg = dict(C=C, H=56, W=W, M=M, k=3, stride=1, pad=1, groups=1)
    c, x, w, b, dy = cg_synth.conv_layer_tensors("six_chunks", B, seed=B * 100 + M, cfg=cfg)
    d = cg.conv_desc(B, C, 56, W, M, 3, stride=1, pad=1, groups=1)
    od = odesc(B, C, 56, W, M, 3, 1, 1, 1)
    cg.cg_profile_enable(True)
    try:
        y = host(conv_fwd(d, dev(x), dev(w), dev(b)))
        dx = host(conv_bwd_data(d, dev(dy), dev(w)))
        names = [cg.cg_profile_get(i)["kernel"] for i in range(cg.cg_profile_count())]
    finally:
        cg.cg_profile_enable(False)
    assert len([n for n in names if n.startswith("igemm_patch_kernel") and n.endswith(",6>")]) == (2 if C > 48 else 1), names
    assert max_abs_rel(y, orc32.conv_fwd(od, x, w, b)) <= TOL
    assert max_abs_rel(dx, orc32.conv_bwd_data(od, dy, w)) <= TOL


def test_patch_and_gather_kernels_agree(orc32):
    """The same forward convolution through both kernels: equal up to summation order."""
    d, od, x, w, b, dy = _setup_patch("p3x3_13_c32_m128")
    a = host(conv_fwd(d, dev(x), dev(w), dev(b)))
    cg.cg_debug_patch_min_tiles(1)
    try:
        c = host(conv_fwd(d, dev(x), dev(w), dev(b)))
    finally:
        cg.cg_debug_patch_min_tiles(512)
    assert max_abs_rel(c, a) <= 1e-5


# Backward-weight through the band kernel (input staged as padded rows): whole-image bands (13x13),
# several bands per image (27x27 with a 5x5 window; 30x30), stride 2, groups, ragged rows and
# columns, a channel count that leaves the last block of columns half empty.
BAND_SHAPES = {
    "b3x3_13_c32_m128": (3, dict(C=32, H=13, M=128, k=3, stride=1, pad=1, groups=1)),
    "b3x3_13_g2_m384": (2, dict(C=48, H=13, M=384, k=3, stride=1, pad=1, groups=2)),
    "b5x5_27_g2_c48": (2, dict(C=48, H=27, M=64, k=5, stride=1, pad=2, groups=2)),
    "b3x3_30_bands": (2, dict(C=20, H=30, M=40, k=3, stride=1, pad=1, groups=1)),
    "b3x3_s2_p1": (2, dict(C=16, H=31, M=32, k=3, stride=2, pad=1, groups=1)),
    "b3x3_nopad_w21": (2, dict(C=7, H=15, W=21, M=100, k=3, stride=1, pad=0, groups=1)),
    "b4x4_p2": (2, dict(C=9, H=16, M=24, k=4, stride=1, pad=2, groups=1)),
}


@pytest.mark.parametrize("name", list(BAND_SHAPES))
def test_band_kernel_backward_weight(orc32, name):
    B, cfg = BAND_SHAPES[name]
    c, x, w, b, dy = cg_synth.conv_layer_tensors(name, B, seed=sum(map(ord, name)), cfg=cfg)
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], Wd, c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    cg.cg_debug_band_kernel(True)                  # off by default: the gathered kernel is what a net runs
    try:
        gdw, gdb = conv_bwd_weight(d, dev(x), dev(dy))
        gdw, gdb = host(gdw), host(gdb)
    finally:
        cg.cg_debug_band_kernel(False)
    assert np.isfinite(gdw).all()
    assert max_abs_rel(gdw, rdw) <= TOL
    assert max_abs_rel(gdb, rdb) <= TOL
    # the gathered kernel on the same problem: equal up to summation order
    hdw, _ = conv_bwd_weight(d, dev(x), dev(dy))
    assert max_abs_rel(host(hdw), gdw) <= 1e-5
