"""Randomised whole-iteration test: 32 seeded random nets (convolutions with groups, strides and
paddings, rectifiers in and out of the positions where they are folded, LRN, max-pooling, an
optional two-branch block joined by a concat, dropout, fully-connected layers, softmax loss), one
training iteration each against the oracle: loss, every materialised activation, the stored
max-pool winners (exact), every local gradient and the updated model (bit-exact from the GPU's own
gradient)."""
import numpy as np
import pytest

import cg_synth
from test_gpu_fullsize import _check_step

pytestmark = pytest.mark.gpu
N_NETS = 32


def _random_net(i):
    rng = np.random.default_rng(7000 + i)
    C, H, W = int(rng.choice([1, 3, 4, 8])), int(rng.integers(9, 20)), int(rng.integers(9, 20))
    in_shape = (C, H, W)
    layers = []

    def add(ly):
        layers.append(ly)
        return len(layers) - 1

    def shape_of(t):
        return in_shape if t < 0 else cg_synth.infer_shapes(layers, in_shape)[t]

    def conv_from(t, relu=True):
        c, h, w = shape_of(t)
        k = int(rng.choice([1, 3, 3, 5]))
        k = min(k, h, w) if min(h, w) < k else k
        if k % 2 == 0:
            k -= 1
        s = int(rng.choice([1, 1, 1, 2])) if min(h, w) >= 2 * k else 1
        p = int(rng.integers(0, k // 2 + 1))
        g = int(rng.choice([1, 1, 2])) if c % 2 == 0 else 1
        M = int(rng.choice([4, 6, 16, 24, 40])) * g
        t = add(dict(kind="conv", inputs=[t], M=M, k=k, stride=s, pad=p, groups=g))
        if relu:
            t = add(dict(kind="relu", inputs=[t]))
        return t

    t = -1
    for _ in range(int(rng.integers(1, 4))):
        t = conv_from(t, relu=rng.random() < 0.85)
        c, h, w = shape_of(t)
        if rng.random() < 0.5:
            size = int(rng.choice([3, 5, 5, 7, 4]))
            t = add(dict(kind="lrn", inputs=[t], size=size, alpha=1e-2, beta=0.75 if size != 7 else 0.6, kappa=1.0))
        if min(h, w) >= 4 and rng.random() < 0.6:
            k, s = [(3, 2), (3, 2), (2, 2), (3, 1), (4, 3)][int(rng.integers(0, 5))]
            p = int(rng.integers(0, 2)) if k >= 3 else 0
            t = add(dict(kind="maxpool", inputs=[t], k=k, stride=s, pad=p))
    if rng.random() < 0.5:                       # two branches from the same tensor, joined along the channels
        c, h, w = shape_of(t)
        a = add(dict(kind="conv", inputs=[t], M=int(rng.choice([4, 8])), k=1, stride=1, pad=0, groups=1))
        a = add(dict(kind="relu", inputs=[a]))
        b = add(dict(kind="conv", inputs=[t], M=int(rng.choice([6, 16])), k=3 if min(h, w) >= 3 else 1, stride=1,
                     pad=1 if min(h, w) >= 3 else 0, groups=1))
        b = add(dict(kind="relu", inputs=[b]))
        branches = [a, b]
        if min(h, w) >= 3 and rng.random() < 0.5:        # a pooling branch as in an inception module
            q = add(dict(kind="maxpool", inputs=[t], k=3, stride=1, pad=1))
            q = add(dict(kind="conv", inputs=[q], M=int(rng.choice([4, 8])), k=1, stride=1, pad=0, groups=1))
            branches.append(add(dict(kind="relu", inputs=[q])))
        t = add(dict(kind="concat", inputs=branches))
    if rng.random() < 0.3:
        t = add(dict(kind="avgpool", inputs=[t]))
    classes = int(rng.integers(3, 12))
    if rng.random() < 0.7:
        t = add(dict(kind="fc", inputs=[t], out=int(rng.choice([16, 33, 64]))))
        t = add(dict(kind="relu", inputs=[t]))
        if rng.random() < 0.6:
            t = add(dict(kind="dropout", inputs=[t], p=0.5))
    t = add(dict(kind="fc", inputs=[t], out=classes))
    add(dict(kind="softmax_ce", inputs=[t]))
    B, K = int(rng.integers(1, 18)), int(rng.integers(0, 5))
    return layers, in_shape, classes, B, K


@pytest.mark.parametrize("i", range(N_NETS))
def test_random_net_iteration(orc32, i):
    layers, in_shape, classes, B, K = _random_net(i)
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=9000 + i, num_classes=classes, init="fan_in", peer_std=1e-3)
    _check_step(orc32, layers, in_shape, B, t)


@pytest.mark.parametrize("i", range(N_NETS))
def test_random_net_schedules_agree_bit_for_bit(i):
    """Three iterations of the three-stream schedule and of the one-stream schedule end in the same
    model, history, local gradients and loss, bit for bit (synchronous semantics, section 2.2)."""
    import torch
    import paper_1706_00095_amd as cg
    from net_util import GpuNet
    layers, in_shape, classes, B, K = _random_net(i)
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=9000 + i, num_classes=classes, init="fan_in", peer_std=1e-3)
    sgd = (0.01, 0.9, 5e-4, 1.0)
    a, b = GpuNet(layers, in_shape, B, t), GpuNet(layers, in_shape, B, t)
    for _ in range(3):
        a.step(sgd, cg.CG_STEP_OVERLAP)
        b.step(sgd, cg.CG_STEP_SERIAL)
    a.sync(); b.sync()
    assert torch.equal(a.loss[:1], b.loss[:1])
    for li in a.w:
        assert torch.equal(a.w[li], b.w[li]) and torch.equal(a.v[li], b.v[li]) and torch.equal(a.g[li], b.g[li]), li
