"""Exact parity of the three convolution passes: small-integer inputs.

With x, w, bias and dy drawn from the integers -3..3 every product and every partial sum is an
integer far below 2^24, which fp32 represents exactly.  Whatever order a kernel adds in -- matrix-core
tiles, K slices added afterwards, taps walked channel block by channel block -- the result must then
equal the oracle's (the definition, accumulated in double and rounded once: exact as well) in every
element, so a tap that is dropped, read twice or taken from the wrong place cannot hide inside a
tolerance.  Every kernel family is driven, and which family ran is read back from the launch log.
The five AlexNet-shaped layers are compared this way at the benchmark's batch of 256, all elements.
"""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_data, conv_bwd_weight, conv_fwd, dev, host
from net_util import GpuNet
from oracle.cgo import conv_desc as odesc
from test_gpu_conv import BAND_SHAPES, PATCH_SHAPES, SHAPES

pytestmark = pytest.mark.gpu

EXTRA_SHAPES = {
    # strided backward-data as a stride-1 problem with 6 x 6 taps and 8 rows (2 channels x 4 phases)
    "eleven_s2": (2, dict(C=4, H=29, M=8, k=11, stride=2, pad=3, groups=2)),
    # fewer than 8 (channel, phase) rows: backward-data by stride phase, and, with more than four taps per
    # dimension and phase, by the one-thread-per-element kernel
    "phase_s2_c1": (3, dict(C=1, H=17, M=12, k=3, stride=2, pad=1, groups=1)),
    "phase_s3_c2_g2": (2, dict(C=2, H=20, M=6, k=5, stride=3, pad=2, groups=2)),
    "eleven_s2_c1": (2, dict(C=2, H=29, M=8, k=11, stride=2, pad=3, groups=2)),
    # strided backward-data through the kernel that stages raw rows of dy (16 output channels a group, 3 x 3 taps)
    "strided_patch_s4": (2, dict(C=3, H=51, M=32, k=11, stride=4, pad=2, groups=1)),
    "strided_patch_s2_g2": (3, dict(C=16, H=23, M=64, k=5, stride=2, pad=2, groups=2)),
    # backward-weight reductions cut into 2, ~10 and more than 16 K slices (both finishing kernels)
    "splitk_few": (8, dict(C=32, H=13, M=384, k=3, stride=1, pad=1, groups=1)),
    "splitk_many": (24, dict(C=8, H=13, M=32, k=3, stride=1, pad=1, groups=1)),
    # a 1x1 layer: backward-data reads the filters in place
    "one_by_one_g2": (3, dict(C=64, H=14, M=96, k=1, stride=1, pad=0, groups=2)),
}


def _descs(B, c):
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], Wd, c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    return d, od


def _same(got, ref, what):
    got, ref = np.asarray(got), np.asarray(ref)
    assert got.shape == ref.shape, what
    bad = np.flatnonzero(got.ravel() != ref.ravel())
    assert bad.size == 0, (what, bad.size, bad[:4], got.ravel()[bad[:4]], ref.ravel()[bad[:4]])


def _logged(fn):
    """Runs fn with the launch log on; returns (result, kernel names)."""
    cg.cg_profile_enable(True)
    try:
        out = fn()
        torch.cuda.synchronize()
        names = [cg.cg_profile_get(i)["kernel"] for i in range(cg.cg_profile_count())]
    finally:
        cg.cg_profile_enable(False)
    return out, names


def _all_three(orc32, B, cfg, seed, fwd=True, bwd_data=True, bwd_weight=True, math=None):
    c, x, w, b, dy = cg_synth.conv_layer_int_tensors(cfg, B, seed)
    d, od = _descs(B, c)
    names = []
    if fwd:
        y, n = _logged(lambda: host(conv_fwd(d, dev(x), dev(w), dev(b), math)))
        names += n
        _same(y, orc32.conv_fwd(od, x, w, b), "forward")
    if bwd_data:
        dx, n = _logged(lambda: host(conv_bwd_data(d, dev(dy), dev(w), math)))
        names += n
        _same(dx, orc32.conv_bwd_data(od, dy, w), "backward-data")
    if bwd_weight:
        (dw, db), n = _logged(lambda: tuple(host(t) for t in conv_bwd_weight(d, dev(x), dev(dy), math)))
        names += n
        rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
        _same(dw, rdw, "backward-weight")
        _same(db, rdb, "bias gradient")
    return d, names


@pytest.mark.parametrize("name", list(SHAPES) + list(EXTRA_SHAPES))
def test_gathered_and_strided_kernels_exact(orc32, name):
    B, cfg = {**SHAPES, **EXTRA_SHAPES}[name]
    if name.startswith("strided_patch"):
        cg.cg_debug_patch_min_tiles(1)
    try:
        d, names = _all_three(orc32, B, cfg, seed=sum(map(ord, name)))
    finally:
        cg.cg_debug_patch_min_tiles(512)
    if name.startswith("strided_patch"):
        assert len([n for n in names if n.startswith("igemm_patch")]) >= 1, names
    else:
        assert all(n.startswith("igemm_kernel") for n in names), names
    if name.startswith("splitk"):
        # the reduction over pixels was cut: partial planes in the workspace, added by a second kernel
        bias_bytes = 4 * d.M * min(d.N, -(-2048 // d.M))
        planes = (cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT) - bias_bytes) // (4 * d.M * d.C * d.KH * d.KW)
        assert planes >= (16 if "many" in name else 2), planes


def test_small_layer_bias_gradient_rides_in_the_k_slice_launch(orc32):
    """Backward-weight of a small layer whose reduction is cut into K slices: two launches in all (the
    matrix kernel and the one that adds the slices, whose extra blocks sum the bias gradient), db exact;
    a layer too large for one block per channel keeps its own bias launches."""
    B, cfg = EXTRA_SHAPES["splitk_few"]
    c, x, w, b, dy = cg_synth.conv_layer_int_tensors(cfg, B, 77)
    d, od = _descs(B, c)
    dx_, dyd = dev(x), dev(dy)
    conv_bwd_weight(d, dx_, dyd)
    torch.cuda.synchronize()
    n0 = cg.cg_debug_launch_count()
    dw, db = conv_bwd_weight(d, dx_, dyd)
    torch.cuda.synchronize()
    assert cg.cg_debug_launch_count() - n0 == 2
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    _same(host(dw), rdw, "backward-weight")
    _same(host(db), rdb, "bias gradient")
    big = cg.conv_desc(64, 32, 27, 27, 64, 3, stride=1, pad=1, groups=1)         # 64 * 729 pixels a channel: two-phase sums
    xb = torch.zeros((64, 32, 27, 27), device="cuda")
    dyb = torch.ones((64, 64, 27, 27), device="cuda")
    n0 = cg.cg_debug_launch_count()
    _, dbb = conv_bwd_weight(big, xb, dyb)
    torch.cuda.synchronize()
    assert cg.cg_debug_launch_count() - n0 == 4
    assert bool((dbb == 64 * 729).all())


@pytest.fixture
def patch_path():
    cg.cg_debug_patch_min_tiles(1)
    yield
    cg.cg_debug_patch_min_tiles(512)


@pytest.mark.parametrize("name", list(PATCH_SHAPES))
def test_patch_kernels_exact(orc32, patch_path, name):
    B, cfg = PATCH_SHAPES[name]
    d, names = _all_three(orc32, B, cfg, seed=sum(map(ord, name)), bwd_data=cfg["stride"] == 1, bwd_weight=False)
    # forward always; backward-data where the output channels of a group (its reduction) come in blocks of 16
    expect = 1 + (1 if cfg["stride"] == 1 and (cfg["M"] // cfg["groups"]) % 16 == 0 else 0)
    assert len([n for n in names if n.startswith("igemm_patch")]) == expect, names
    if cfg["M"] <= 48:
        assert any(n.startswith("igemm_patch16_kernel") for n in names), names


@pytest.mark.parametrize("B,M,groups,resident", [(3, 128, 1, 3), (5, 384, 2, 12), (7, 256, 1, 6)])
def test_patch_kernel_two_launches_exact(orc32, patch_path, B, M, groups, resident):
    cfg = dict(C=32, H=13, M=M, k=3, stride=1, pad=1, groups=groups)
    cg.cg_debug_resident_blocks(resident)
    try:
        d, names = _all_three(orc32, B, cfg, seed=B * 1000 + M, bwd_data=False, bwd_weight=False)
    finally:
        cg.cg_debug_resident_blocks(512)
    assert len([n for n in names if n.startswith("igemm_patch_kernel")]) == 2, names


@pytest.mark.parametrize("B,C,M,W", [(2, 16, 64, 56), (1, 64, 160, 56), (2, 32, 128, 52)])
def test_patch_kernel_six_chunks_exact(orc32, patch_path, B, C, M, W):
    cfg = dict(C=C, H=56, W=W, M=M, k=3, stride=1, pad=1, groups=1)
    d, names = _all_three(orc32, B, cfg, seed=B * 100 + M, bwd_weight=False)
    assert len([n for n in names if n.startswith("igemm_patch_kernel") and n.endswith(",6>")]) == (2 if C > 48 else 1), names
    if C <= 48:       # backward-data with at most 48 rows: the 16-row-tile kernel, six chunks as well
        assert any(n.startswith("igemm_patch16_kernel") and n.endswith(",6>") for n in names), names


@pytest.mark.parametrize("name", list(BAND_SHAPES))
def test_band_kernel_exact(orc32, name):
    B, cfg = BAND_SHAPES[name]
    cg.cg_debug_band_kernel(True)
    try:
        d, names = _all_three(orc32, B, cfg, seed=sum(map(ord, name)), fwd=False, bwd_data=False)
    finally:
        cg.cg_debug_band_kernel(False)
    # one shape's last band of rows is shorter than the band kernel's pipeline needs: the gathered kernel takes it
    family = "igemm_kernel" if name == "b3x3_s2_p1" else "igemm_wgrad_kernel"
    assert names and all(n.startswith(family) for n in names), names


@pytest.mark.parametrize("B,IN,OUT", [(5, 37, 11), (64, 256, 1000), (130, 513, 70)])
def test_fully_connected_forward_exact_with_bias(orc32, B, IN, OUT):
    """y[b][o] = bias[o] + sum_i x[b][i] W[o][i] on integers: the per-column bias of the matrix kernels'
    store (and of the K-slice finishing kernel) and the rectifier folded behind it, all elements."""
    rng = np.random.default_rng(B * 7 + OUT)
    layers = [dict(kind="fc", inputs=[-1], out=OUT), dict(kind="relu", inputs=[0]),
              dict(kind="fc", inputs=[1], out=3), dict(kind="softmax_ce", inputs=[2])]
    in_shape = (IN, 1, 1)
    t = cg_synth.net_tensors(layers, in_shape, B, 1, seed=B, num_classes=3)
    t["x"] = rng.integers(-3, 4, size=(B, IN, 1, 1)).astype(np.float32)
    t["buckets"][0] = rng.integers(-3, 4, size=OUT * IN + OUT).astype(np.float32)
    gn = GpuNet(layers, in_shape, B, t)
    gn.step((0.01, 0.9, 5e-4, 1.0))
    gn.sync()
    W_, b = t["buckets"][0][:OUT * IN].reshape(OUT, IN), t["buckets"][0][OUT * IN:]
    assert np.abs(b).max() > 0
    ref = orc32.relu_fwd(orc32.fc_fwd(t["x"].reshape(B, IN), W_, b))
    assert gn.fused(0)
    _same(host(gn.act(1)).reshape(B, OUT), ref, "fc forward + bias + rectifier")


@pytest.mark.parametrize("layer", list(cg_synth.ALEXNET_CONVS))
def test_alexnet_conv_layer_at_b256_exact(orc32, layer):
    """Configuration 2 at its real size, in the launch configuration the benchmark times: every element
    of y, dx, dw and db.  Backward-weight sums 256 * OH * OW <= 774 400 products of magnitude <= 9."""
    cfg = cg_synth.ALEXNET_CONVS[layer]
    d, names = _all_three(orc32, 256, cfg, seed=100 + list(cg_synth.ALEXNET_CONVS).index(layer))
    if layer != "conv1":
        assert any(n.startswith("igemm_patch") for n in names), names
