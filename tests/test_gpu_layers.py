"""GPU parity of the glue layers inside small nets the oracle runs in full: LRN windows the
streaming kernel specialises (3, 5, 7) and one it does not (4), max-pool windows with and
without specialisation and with padding, and rectifiers in positions where their forward is
folded into the producer's store and their backward into the consumer's kernel."""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import host, max_abs_rel
from net_util import GpuNet
from oracle import net as onet

pytestmark = pytest.mark.gpu
TOL = 1e-3
SGD = (0.01, 0.9, 5e-4, 1.0)


def _net(lrn_size, pool, in_shape=(6, 14, 14)):
    k, s, p = pool
    layers = [
        dict(kind="conv", inputs=[-1], M=20, k=3, stride=1, pad=1, groups=1),
        dict(kind="relu", inputs=[0]),
        dict(kind="lrn", inputs=[1], size=lrn_size, alpha=1e-2, beta=0.75 if lrn_size != 7 else 0.6, kappa=1.0),
        dict(kind="maxpool", inputs=[2], k=k, stride=s, pad=p),
        dict(kind="conv", inputs=[3], M=16, k=3, stride=1, pad=1, groups=2),
        dict(kind="relu", inputs=[4]),
        dict(kind="maxpool", inputs=[5], k=2, stride=2, pad=0),
        dict(kind="fc", inputs=[6], out=24),
        dict(kind="relu", inputs=[7]),
        dict(kind="dropout", inputs=[8], p=0.5),
        dict(kind="fc", inputs=[9], out=7),
        dict(kind="softmax_ce", inputs=[10]),
    ]
    return layers, in_shape


# the last three: planes of 99, 110 and 225 pixels, whose last group of four pixels (LRN, bias
# gradient) and whose 16-byte staging groups (pooling) are ragged in every possible way
@pytest.mark.parametrize("lrn_size,pool,in_shape", [(3, (3, 2, 0), (6, 14, 14)), (5, (3, 1, 1), (6, 14, 14)),
                                                    (7, (2, 2, 0), (6, 14, 14)), (4, (4, 3, 1), (6, 14, 14)),
                                                    (5, (3, 2, 0), (5, 9, 11)), (3, (3, 2, 1), (7, 10, 11)),
                                                    (5, (3, 1, 1), (3, 15, 15))])
@pytest.mark.parametrize("fuse", [0, 1, 3])
def test_layer_variants_match_oracle(orc32, lrn_size, pool, in_shape, fuse):
    """fuse: the LRN and the max-pool behind it (window sizes 3 and 5) as separate kernels (0), as one
    kernel in forward (1, the default) or in both directions (3)."""
    layers, in_shape = _net(lrn_size, pool, in_shape)
    B = 5
    t = cg_synth.net_tensors(layers, in_shape, B, 2, seed=40 + lrn_size, num_classes=7, init="fan_in", peer_std=1e-3)
    cg.cg_debug_fuse_lrn_pool(fuse)
    try:
        gn = GpuNet(layers, in_shape, B, t)
    finally:
        cg.cg_debug_fuse_lrn_pool(1)
    gn.step(SGD)
    gn.sync()
    buckets = {k: v.copy() for k, v in t["buckets"].items()}
    loss, acts, aux = onet.forward(orc32, layers, t["x"], buckets, t["labels"], t["masks"])
    grads, dact, _ = onet.backward(orc32, layers, t["x"], buckets, t["masks"], acts, aux)
    assert abs(float(host(gn.loss)[0]) - float(loss)) <= TOL * max(1.0, abs(float(loss)))
    folded_fwd = folded_bwd = 0
    for li in range(len(layers) - 1):
        if gn.fused(li):
            folded_fwd += 1
            continue
        assert max_abs_rel(host(gn.act(li)), acts[li].ravel()) <= TOL, ("activation", li, layers[li]["kind"])
    for li, dref in dact.items():
        if li == len(layers) - 1:
            continue
        if gn.grad_folded(li):
            folded_bwd += 1
            continue
        assert max_abs_rel(host(gn.act(li, 1)), dref.ravel()) <= TOL, ("gradient", li, layers[li]["kind"])
    fused = lrn_size in (3, 5)
    # the three rectifiers, both directions, and the LRN where it runs fused with its pool
    assert folded_fwd == 3 + (1 if fuse and fused else 0) and folded_bwd == 3 + (1 if fuse == 3 and fused else 0)
    for li in grads:
        assert max_abs_rel(host(gn.g[li]), grads[li]) <= TOL, ("g_local", li)


@pytest.mark.parametrize("lrn_size,pool,in_shape", [(5, (3, 2, 0), (3, 100, 100)), (3, (3, 1, 1), (2, 90, 100)),
                                                    (5, (4, 3, 1), (2, 130, 70))])
def test_pooling_planes_beyond_the_lds_staging(orc32, lrn_size, pool, in_shape):
    """Planes of 10 000 / 9 000 / 9 100 elements: the pooling kernels read them straight from global
    memory (forward only in the first case, 2 401 outputs a plane; both directions in the second;
    a window without a specialised kernel in the third).  With a million window comparisons a
    last-bit difference in forward can elect another winner, so backward is compared from the
    GPU's own forward state (the winners must then be the oracle's exactly)."""
    from test_gpu_fullsize import _check_step
    layers, in_shape = _net(lrn_size, pool, in_shape)
    t = cg_synth.net_tensors(layers, in_shape, 3, 2, seed=50 + lrn_size, num_classes=7, init="fan_in", peer_std=1e-3)
    _check_step(orc32, layers, in_shape, 3, t)


@pytest.mark.parametrize("mode", [0, 3])
def test_alexnet_shaped_iteration_lrn_pool_modes(orc32, mode):
    """The AlexNet-shaped net (B = 16) with its two LRN + max-pool pairs as four separate kernels (0) and
    with both directions fused (3); the default, forward fused only, is what every other whole-net
    test runs.  Planes of 55 x 55 (four row bands a channel) and 27 x 27 (one)."""
    from test_gpu_fullsize import _check_step
    layers, in_shape = cg_synth.alexnet_layers()
    t = cg_synth.net_tensors(layers, in_shape, 16, 1, seed=4, num_classes=1000)
    cg.cg_debug_fuse_lrn_pool(mode)
    try:
        gn = _check_step(orc32, layers, in_shape, 16, t)
    finally:
        cg.cg_debug_fuse_lrn_pool(1)
    lrn = [i for i, ly in enumerate(layers) if ly["kind"] == "lrn"]
    assert [cg.cg_net_layer_fused(gn.net, i) for i in lrn] == [mode, mode]


def test_measurement_kernels_run():
    """The ceiling probes of the benchmark (streaming kernels, matrix-pipeline loop) launch and finish;
    the copy variant copies."""
    a = torch.arange(4096, dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    cg.cg_debug_stream(b, a, a, a.numel() * 4, 0)
    out = torch.empty(256 * 3, device="cuda")
    cg.cg_debug_mfma_loop(out, 3, 7)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and bool(torch.isfinite(out).all())
    with pytest.raises(Exception):
        cg.cg_debug_mfma_loop(out, 0, 7)
