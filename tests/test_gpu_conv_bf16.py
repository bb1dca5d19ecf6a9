"""The optional bf16 matrix-core path (cg_conv_*_math, CG_STEP_BF16 / CG_STEP_BF16X3) against the same
oracle as the fp32 path.

 CG_MATH_BF16   : operands rounded to bf16, fp32 accumulation: max-abs-relative error <= 2e-2.
 CG_MATH_BF16X3 : operands split into two bf16 numbers, three products: <= 1e-4 here (the fp32 bound
                  is 1e-3; what the mode drops is about 2^-16 of a product).
Small integers are exact in bf16, so on integer inputs both modes must equal the oracle in every
element: that pins which reduction index a lane puts into which slot of the 16-deep bf16 matrix
instruction, on every kernel family the modes run.
"""
import numpy as np
import pytest

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_data, conv_bwd_weight, conv_fwd, dev, host, max_abs_rel
from net_util import GpuNet
from oracle import net as onet
from oracle.cgo import conv_desc as odesc
from test_gpu_conv import PATCH_SHAPES, SHAPES
from test_gpu_conv_exact import EXTRA_SHAPES, _all_three
from test_gpu_fullsize import _backward_state_from_gpu_forward, _check_step
from test_oracle_net import _small_alexnet_like

pytestmark = pytest.mark.gpu
MODES = {"bf16": (cg.CG_MATH_BF16, 2e-2), "bf16x3": (cg.CG_MATH_BF16X3, 1e-4)}
SGD = (0.01, 0.9, 5e-4, 1.0)
# backward-data of these exists in fp32 only (fewer than 8 (channel, stride phase) rows: vector kernels)
FP32_ONLY_BWD_DATA = {"phase_s2_c1", "phase_s3_c2_g2", "eleven_s2_c1"}


def _tagged(names, tag):
    return names and all(n.endswith("," + tag + ">") for n in names)


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("name", list(SHAPES) + list(EXTRA_SHAPES))
def test_exact_on_integers_gathered(orc32, name, mode):
    B, cfg = {**SHAPES, **EXTRA_SHAPES}[name]
    if name.startswith("strided_patch"):
        cg.cg_debug_patch_min_tiles(1)
    try:
        d, names = _all_three(orc32, B, cfg, seed=sum(map(ord, name)), bwd_data=name not in FP32_ONLY_BWD_DATA,
                              math=MODES[mode][0])
    finally:
        cg.cg_debug_patch_min_tiles(512)
    assert _tagged(names, mode), names


def test_fp32_only_backward_data_is_refused_not_silently_computed():
    B, cfg = EXTRA_SHAPES["phase_s2_c1"]
    c, x, w, b, dy = cg_synth.conv_layer_int_tensors(cfg, B, 1)
    d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    with pytest.raises(cg.CgError) as e:
        conv_bwd_data(d, dev(dy), dev(w), cg.CG_MATH_BF16)
    assert e.value.code == cg.CG_EUNSUPPORTED
    with pytest.raises(cg.CgError) as e:
        conv_fwd(d, dev(x), dev(w), dev(b), 7)
    assert e.value.code == cg.CG_EINVAL


@pytest.fixture
def patch_path():
    cg.cg_debug_patch_min_tiles(1)
    yield
    cg.cg_debug_patch_min_tiles(512)


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("name", list(PATCH_SHAPES))
def test_exact_on_integers_patch(orc32, patch_path, name, mode):
    B, cfg = PATCH_SHAPES[name]
    d, names = _all_three(orc32, B, cfg, seed=sum(map(ord, name)), bwd_data=cfg["stride"] == 1, bwd_weight=False,
                          math=MODES[mode][0])
    assert _tagged(names, mode), names
    assert names[0].startswith("igemm_patch_kernel"), names       # no 16-row-tile instance in these modes: 64-row tiles


@pytest.mark.parametrize("mode", list(MODES))
def test_exact_on_integers_six_chunks(orc32, patch_path, mode):
    cfg = dict(C=64, H=56, W=56, M=160, k=3, stride=1, pad=1, groups=1)
    d, names = _all_three(orc32, 1, cfg, seed=77, bwd_weight=False, math=MODES[mode][0])
    assert len([n for n in names if n.startswith("igemm_patch_kernel") and ",6," in n]) == 2, names


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("name", list(SHAPES))
def test_within_the_mode_s_bound_on_normal_inputs(orc32, name, mode):
    math, tol = MODES[mode]
    B, cfg = SHAPES[name]
    c, x, w, b, dy = cg_synth.conv_layer_tensors(name, B, seed=sum(map(ord, name)), cfg=cfg)
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], Wd, c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    assert max_abs_rel(host(conv_fwd(d, dev(x), dev(w), dev(b), math)), orc32.conv_fwd(od, x, w, b)) <= tol
    assert max_abs_rel(host(conv_bwd_data(d, dev(dy), dev(w), math)), orc32.conv_bwd_data(od, dy, w)) <= tol
    gdw, gdb = conv_bwd_weight(d, dev(x), dev(dy), math)
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    assert max_abs_rel(host(gdw), rdw) <= tol and max_abs_rel(host(gdb), rdb) <= 1e-5       # the bias sum stays fp32


def test_bf16_really_rounds_and_bf16x3_does_not(orc64):
    """The two modes are what they say: on normal inputs plain bf16 is off by about 2^-9 per operand, the
    split mode by about 2^-16 -- not the same kernel under two names, and not fp32 under either."""
    B, cfg = SHAPES["conv3_like"]
    c, x, w, b, dy = cg_synth.conv_layer_tensors("conv3_like", B, seed=5, cfg=cfg)
    d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], c["H"], c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    ref = orc64.conv_fwd(od, x.astype(np.float64), w.astype(np.float64), b.astype(np.float64))
    e32 = max_abs_rel(host(conv_fwd(d, dev(x), dev(w), dev(b))), ref)
    e16 = max_abs_rel(host(conv_fwd(d, dev(x), dev(w), dev(b), cg.CG_MATH_BF16)), ref)
    ex3 = max_abs_rel(host(conv_fwd(d, dev(x), dev(w), dev(b), cg.CG_MATH_BF16X3)), ref)
    assert 2e-4 < e16 < 2e-2, e16
    assert e32 < 2e-6 and e32 < ex3 < 1e-4 and ex3 < e16 / 20, (e32, ex3, e16)


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("layer", list(cg_synth.ALEXNET_CONVS))
def test_alexnet_layers_full_spatial_size(orc32, layer, mode):
    """Every AlexNet-shaped layer at its real geometry (B = 4), element by element, all three passes."""
    math, tol = MODES[mode]
    B = 4
    c, x, w, b, dy = cg_synth.conv_layer_tensors(layer, B, seed=2)
    d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    od = odesc(B, c["C"], c["H"], c["H"], c["M"], c["k"], c["stride"], c["pad"], c["groups"])
    dx_, dw_, db_, dy_ = dev(x), dev(w), dev(b), dev(dy)
    assert max_abs_rel(host(conv_fwd(d, dx_, dw_, db_, math)), orc32.conv_fwd(od, x, w, b)) <= tol
    assert max_abs_rel(host(conv_bwd_data(d, dy_, dw_, math)), orc32.conv_bwd_data(od, dy, w)) <= tol
    rdw, rdb = orc32.conv_bwd_weight(od, x, dy)
    gdw, gdb = conv_bwd_weight(d, dx_, dy_, math)
    assert max_abs_rel(host(gdw), rdw) <= tol and max_abs_rel(host(gdb), rdb) <= 1e-5


@pytest.mark.parametrize("layer,mode", [("conv2", "bf16"), ("conv4", "bf16"), ("conv1", "bf16x3"), ("conv3", "bf16x3")])
def test_alexnet_layer_at_b256_exact_on_integers(orc32, layer, mode):
    """At the benchmark's size, in the launch configuration the benchmark's bf16 lines time."""
    d, names = _all_three(orc32, 256, cg_synth.ALEXNET_CONVS[layer], seed=300 + len(layer), math=MODES[mode][0])
    assert _tagged(names, mode), names


NETS = {
    "tiny_cnn_cfg1": lambda: cg_synth.tiny_cnn_layers() + (10, 8, 4, "xavier", 1e-2, 0),
    "alexnet_like": lambda: _small_alexnet_like() + (7, 6, 4, "fan_in", 1e-3, 4),
    "inception": lambda: cg_synth.inception_layers(modules=2, cin=12, hw=6, num_classes=9) + (9, 5, 8, "fan_in", 1e-3, 5),
    "alexnet_b16": lambda: cg_synth.alexnet_layers() + (1000, 16, 1, "fan_in", 1e-3, 4),
}


@pytest.mark.parametrize("name", list(NETS))
def test_whole_iteration_bf16x3_meets_the_fp32_bound(orc32, name):
    layers, in_shape, ncls, B, K, init, pstd, seed = NETS[name]()
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=seed, num_classes=ncls, init=init, peer_std=pstd)
    _check_step(orc32, layers, in_shape, B, t, flags=cg.CG_STEP_BF16X3)


@pytest.mark.parametrize("name", list(NETS))
def test_whole_iteration_bf16_layer_by_layer(orc32, name):
    """CG_STEP_BF16: the 2e-2 bound is a bound per contraction, so every convolution and fully-connected
    layer is checked on its own, the oracle's layer applied to the tensors the GPU step itself fed it:
    forward output (with the folded rectifier), weight and bias gradient.  The update stays bit-exact."""
    tol = 2e-2
    layers, in_shape, ncls, B, K, init, pstd, seed = NETS[name]()
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=seed, num_classes=ncls, init=init, peer_std=pstd)
    gn = GpuNet(layers, in_shape, B, t)
    gn.step(SGD, cg.CG_STEP_BF16)
    gn.sync()
    shapes = cg_synth.infer_shapes(layers, in_shape)
    checked = 0
    for li, ly in enumerate(layers):
        if ly["kind"] not in ("conv", "fc"):
            continue
        src = ly["inputs"][0]
        xin = t["x"] if src < 0 else host(gn.act(src)).reshape((B,) + tuple(shapes[src]))
        bucket = t["buckets"][li]
        out_li = li + 1 if gn.fused(li) else li           # a folded rectifier's output stands for the layer's
        got = host(gn.act(out_li)).reshape((B,) + tuple(shapes[li]))
        dy = host(gn.act(li, 1)).reshape((B,) + tuple(shapes[li]))
        if ly["kind"] == "conv":
            N, C, H, W = xin.shape
            od = odesc(N, C, H, W, ly["M"], ly["k"], ly["stride"], ly["pad"], ly["groups"])
            nw = ly["M"] * (C // ly["groups"]) * ly["k"] * ly["k"]
            w = bucket[:nw].reshape(ly["M"], C // ly["groups"], ly["k"], ly["k"])
            ref = orc32.conv_fwd(od, xin, w, bucket[nw:])
            rdw, rdb = orc32.conv_bwd_weight(od, xin, dy)
        else:
            x2 = xin.reshape(B, -1)
            nw = ly["out"] * x2.shape[1]
            ref = orc32.fc_fwd(x2, bucket[:nw].reshape(ly["out"], -1), bucket[nw:]).reshape(got.shape)
            rdw, rdb = orc32.fc_bwd_weight(x2, dy.reshape(B, -1))
        if gn.fused(li):
            ref = orc32.relu_fwd(ref)
        assert max_abs_rel(got, ref) <= tol, ("forward", li)
        g = host(gn.g[li])
        assert max_abs_rel(g[:nw], rdw.ravel()) <= tol, ("weight gradient", li)
        assert max_abs_rel(g[nw:], rdb.ravel()) <= 1e-4, ("bias gradient", li)
        w0, v0 = bucket.copy(), np.zeros_like(bucket)
        orc32.grad_reduce_sgd(w0, v0, g, t["peers"][li], *SGD)
        assert host(gn.w[li]).tobytes() == w0.tobytes() and host(gn.v[li]).tobytes() == v0.tobytes()
        checked += 1
    assert checked >= 3
