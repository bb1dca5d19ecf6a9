"""Pins for the oracle's whole-iteration composition (forward, backward in inverse layer
order, per-layer update): finite differences of the scalar loss with respect to every
parameter tensor on the double build, closed-form losses, and the update invariants."""
import math

import numpy as np
import pytest

import cg_synth
from oracle import net as onet


def _small_alexnet_like():
    """All AlexNet layer kinds on a small image: grouped conv, LRN, overlapping pool, dropout."""
    L = [
        dict(kind="conv", inputs=[-1], M=8, k=5, stride=2, pad=0, groups=1),
        dict(kind="relu", inputs=[0]),
        dict(kind="lrn", inputs=[1], size=5, alpha=0.5, beta=0.75, kappa=1.0),
        dict(kind="maxpool", inputs=[2], k=3, stride=2, pad=0),
        dict(kind="conv", inputs=[3], M=8, k=3, stride=1, pad=1, groups=2),
        dict(kind="relu", inputs=[4]),
        dict(kind="fc", inputs=[5], out=12),
        dict(kind="relu", inputs=[6]),
        dict(kind="dropout", inputs=[7], p=0.5),
        dict(kind="fc", inputs=[8], out=7),
        dict(kind="softmax_ce", inputs=[9]),
    ]
    return L, (3, 19, 19)


NETS = {
    "tiny_cnn": lambda: cg_synth.tiny_cnn_layers() + (10,),
    "alexnet_like": lambda: _small_alexnet_like() + (7,),
    "inception": lambda: cg_synth.inception_layers(modules=2, cin=12, hw=6, num_classes=9) + (9,),
}


def _to64(t):
    return dict(x=t["x"].astype(np.float64), labels=t["labels"],
                buckets={k: v.astype(np.float64) for k, v in t["buckets"].items()},
                peers={k: [p.astype(np.float64) for p in v] for k, v in t["peers"].items()},
                masks=t["masks"])


@pytest.mark.parametrize("name", list(NETS))
def test_parameter_gradients_by_finite_differences(orc64, name):
    layers, in_shape, ncls = NETS[name]()
    B = 3 if name != "tiny_cnn" else 2
    t = _to64(cg_synth.net_tensors(layers, in_shape, B, 0, seed=7, num_classes=ncls, init="xavier"))
    rng = np.random.default_rng(70)
    for li in t["buckets"]:       # give the biases a value so their path is exercised
        t["buckets"][li] += rng.standard_normal(t["buckets"][li].size) * 0.05
    loss, acts, aux = onet.forward(orc64, layers, t["x"], t["buckets"], t["labels"], t["masks"])
    grads, _, dxin = onet.backward(orc64, layers, t["x"], t["buckets"], t["masks"], acts, aux, need_input_grad=True)
    assert set(grads) == set(t["buckets"])
    h = 1e-6

    def L():
        return float(onet.loss_only(orc64, layers, t["x"], t["labels"], t["buckets"], t["masks"]))

    for li, b in t["buckets"].items():
        idx = np.concatenate([rng.choice(b.size, size=min(6, b.size), replace=False), [b.size - 1]])
        for i in idx:
            keep = b[i]
            b[i] = keep + h; lp = L()
            b[i] = keep - h; lm = L()
            b[i] = keep
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grads[li][i]) <= 2e-6 * max(abs(fd), 1e-3), (name, li, i, fd, grads[li][i])
    # the input gradient covers backward-data of the first layer and the fan-out sums
    xf = t["x"].ravel()
    for i in rng.choice(xf.size, size=6, replace=False):
        keep = xf[i]
        xf[i] = keep + h; lp = L()
        xf[i] = keep - h; lm = L()
        xf[i] = keep
        fd = (lp - lm) / (2 * h)
        assert abs(fd - dxin.ravel()[i]) <= 2e-6 * max(abs(fd), 1e-3)


def test_zero_classifier_gives_log_num_classes(orc32):
    layers, in_shape = cg_synth.tiny_cnn_layers()
    t = cg_synth.net_tensors(layers, in_shape, 8, 0, seed=0, num_classes=10, init="xavier")
    t["buckets"][5][:] = 0
    loss = onet.loss_only(orc32, layers, t["x"], t["labels"], t["buckets"], t["masks"])
    assert abs(float(loss) - math.log(10.0)) < 1e-6


def test_xavier_init_loss_is_near_log10(orc32):
    """Xavier-uniform weights with zero biases (a freshly initialised model): small logits."""
    layers, in_shape = cg_synth.tiny_cnn_layers()
    t = cg_synth.net_tensors(layers, in_shape, 8, 4, seed=0, num_classes=10, init="xavier", peer_std=1e-2, bias_std=0.0)
    loss = onet.loss_only(orc32, layers, t["x"], t["labels"], t["buckets"], t["masks"])
    assert abs(float(loss) - math.log(10.0)) < 0.3


def test_train_step_applies_eq1_per_layer(orc32):
    """After one iteration every bucket equals the solver update of its own local gradient
    plus peers; with lr = 0 and zero history nothing moves."""
    layers, in_shape = cg_synth.tiny_cnn_layers()
    t = cg_synth.net_tensors(layers, in_shape, 8, 4, seed=0, num_classes=10, init="xavier", peer_std=1e-2)
    w0 = {k: v.copy() for k, v in t["buckets"].items()}
    hist = {k: np.zeros_like(v) for k, v in t["buckets"].items()}
    loss, grads = onet.train_step(orc32, layers, t["x"], t["labels"], t["buckets"], hist, t["peers"],
                                  t["masks"], 0.01, 0.9, 5e-4)
    for li in w0:
        s = grads[li].copy()
        for p in t["peers"][li]:
            s = s + p
        vn = np.float32(0.9) * np.zeros_like(s) + np.float32(0.01) * (s + np.float32(5e-4) * w0[li])
        assert np.array_equal(hist[li], vn) and np.array_equal(t["buckets"][li], w0[li] - vn)
    t2 = cg_synth.net_tensors(layers, in_shape, 8, 4, seed=0, num_classes=10, init="xavier", peer_std=1e-2)
    hist2 = {k: np.zeros_like(v) for k, v in t2["buckets"].items()}
    onet.train_step(orc32, layers, t2["x"], t2["labels"], t2["buckets"], hist2, t2["peers"], t2["masks"], 0.0, 0.9, 5e-4)
    for li in w0:
        assert t2["buckets"][li].tobytes() == w0[li].tobytes() and not hist2[li].any()


def test_weight_gradients_do_not_depend_on_pool_tie_break(orc64):
    """Post-ReLU zero ties in a max-pool window route gradient to an element whose ReLU
    derivative is 0, so parameter gradients are the same whichever tied element wins."""
    layers = [
        dict(kind="conv", inputs=[-1], M=4, k=3, stride=1, pad=1, groups=1),
        dict(kind="relu", inputs=[0]),
        dict(kind="maxpool", inputs=[1], k=2, stride=2, pad=0),
        dict(kind="fc", inputs=[2], out=3),
        dict(kind="softmax_ce", inputs=[3]),
    ]
    t = _to64(cg_synth.net_tensors(layers, (2, 6, 6), 4, 0, seed=9, num_classes=3, init="xavier"))
    t["buckets"][0][-4:] = -0.2     # negative bias: many all-zero pooling windows
    loss, acts, aux = onet.forward(orc64, layers, t["x"], t["buckets"], t["labels"], t["masks"])
    assert (acts[2] == 0).any()
    g1, _, _ = onet.backward(orc64, layers, t["x"], t["buckets"], t["masks"], acts, aux)
    am = aux[2].copy()
    zero_win = acts[2] == 0
    am[zero_win] += 1               # move the winner of every all-zero window to its neighbour
    aux2 = list(aux); aux2[2] = am
    g2, _, _ = onet.backward(orc64, layers, t["x"], t["buckets"], t["masks"], acts, aux2)
    for li in g1:
        np.testing.assert_allclose(g1[li], g2[li], atol=1e-15)


def test_googlenet_shaped_layer_list():
    """The second benchmark net of the paper's Table 1 by shape: 7.0 M parameters without the
    auxiliary classifiers, stage widths 256/480, 512/512/512/528/832, 832/1024 on 28, 14 and 7
    pixel planes (Szegedy et al. 2014, Table 1), 2 x 1.58 G multiply-adds per image forward."""
    layers, in_shape, names = cg_synth.googlenet_layers()
    shapes = cg_synth.infer_shapes(layers, in_shape)
    cat = [shapes[i] for i, ly in enumerate(layers) if ly["kind"] == "concat"]
    assert cat == [(256, 28, 28), (480, 28, 28), (512, 14, 14), (512, 14, 14), (512, 14, 14), (528, 14, 14),
                   (832, 14, 14), (832, 7, 7), (1024, 7, 7)]
    pl = cg_synth.param_layers(layers, in_shape)
    assert len(pl) == 58 and sorted(names) == [li for li, _, _ in pl]
    assert sum(int(np.prod(ws)) + nb for _, ws, nb in pl) == 6998552
    macs = sum(int(np.prod(ws)) * shapes[li][1] * shapes[li][2] for li, ws, _ in pl)
    assert abs(macs / 1e9 - 1.58) < 0.01
    assert shapes[0] == (64, 112, 112) and shapes[2] == (64, 56, 56)      # 3x3/2 pool, ceil mode: 112 -> 56


def test_googlenet_shaped_net_gradients_by_finite_differences(orc64):
    """The whole 142-layer composition (fan-out of one tensor into four branches, concat, clipped
    pool windows) on a 64 x 64 input: finite differences on a few parameters of early, middle and
    late layers."""
    layers, in_shape, names = cg_synth.googlenet_layers(num_classes=11, hw=64)
    t = _to64(cg_synth.net_tensors(layers, in_shape, 2, 0, seed=9, num_classes=11, init="xavier"))
    rng = np.random.default_rng(71)
    for li in t["buckets"]:
        t["buckets"][li] += rng.standard_normal(t["buckets"][li].size) * 0.02
    loss, acts, aux = onet.forward(orc64, layers, t["x"], t["buckets"], t["labels"], t["masks"])
    grads, _, _ = onet.backward(orc64, layers, t["x"], t["buckets"], t["masks"], acts, aux)
    by_name = {v: k for k, v in names.items()}
    h = 1e-6
    for nm in ("conv1", "conv2", "3a_5x5_reduce", "4c_3x3", "4e_pool_proj", "5b_1x1", "classifier"):
        b = t["buckets"][by_name[nm]]
        g = grads[by_name[nm]]
        for i in (int(np.argmax(np.abs(g))), b.size - 1):
            keep = b[i]
            b[i] = keep + h; lp = float(onet.loss_only(orc64, layers, t["x"], t["labels"], t["buckets"], t["masks"]))
            b[i] = keep - h; lm = float(onet.loss_only(orc64, layers, t["x"], t["labels"], t["buckets"], t["masks"]))
            b[i] = keep
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[i]) <= 1e-5 * max(abs(fd), 1e-4), (nm, i, fd, g[i])
