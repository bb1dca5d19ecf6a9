"""Parity at the benchmark's real sizes, in the launch configuration bench.py times.

 - the whole AlexNet-shaped net at B = 16, 64 and 256 (the benchmark's workload; the oracle needs
   about half a minute for it) against the oracle element by element;
 - the three fully-connected layers at B=256 as their own net;
 - each AlexNet convolution layer at B=256 on sampled outputs the oracle's definition gives one by
   one, and through the adjoint identities, which hold at any size (every element of these layers is
   compared in test_gpu_conv_exact.py, on integer inputs).
"""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_data, conv_bwd_weight, conv_fwd, dev, host, max_abs_rel
from net_util import GpuNet
from oracle import net as onet

pytestmark = pytest.mark.gpu
TOL = 1e-3
SGD = (0.01, 0.9, 5e-4, 1.0)


def _backward_state_from_gpu_forward(orc32, gn, layers, t, acts):
    """Backward depends on decisions taken in forward (ReLU sign, max-pool winner).  On a deep
    net a forward value that differs in the last bit can flip such a decision, and the two
    backward passes then differ legitimately.  So the oracle's backward is run from the GPU's own
    forward activations: both sides take every decision in fp32 on the same numbers.  The
    max-pool winners the GPU stored must then be exactly the oracle's."""
    acts_g = []
    for li, ly in enumerate(layers[:-1]):
        if ly["kind"] == "lrn" and gn.fused(li):
            # fused with the pool that follows: its output exists nowhere; the oracle's LRN of the GPU's input
            # stands for it
            src = ly["inputs"][0]
            a = t["x"] if src < 0 else acts_g[src]
            acts_g.append(orc32.lrn_fwd(a, ly["size"], ly["alpha"], ly["beta"], ly["kappa"])[0])
        else:
            acts_g.append(host(gn.act(li)).reshape(acts[li].shape))
    acts_g.append(acts[-1])
    aux_g = []
    for li, ly in enumerate(layers):
        src = ly["inputs"][0]
        a = t["x"] if src < 0 else acts_g[src]
        if ly["kind"] == "conv":
            from oracle.cgo import conv_desc
            N, C, H, W = a.shape
            aux_g.append(conv_desc(N, C, H, W, ly["M"], ly["k"], ly["stride"], ly["pad"], ly["groups"]))
        elif ly["kind"] == "lrn":
            aux_g.append(orc32.lrn_fwd(a, ly["size"], ly["alpha"], ly["beta"], ly["kappa"])[1])
        elif ly["kind"] == "maxpool":
            am = orc32.maxpool_fwd(a, ly["k"], ly["stride"], ly["pad"])[1]
            got = host(gn.act(li, 2)).view(np.int32).reshape(am.shape)
            if src >= 0 and layers[src]["kind"] == "lrn" and gn.fused(src):
                # The pooled values come from the GPU's own LRN arithmetic (same definition, other rounding
                # of scale^-beta), so where two values of a window agree to the last bits either may win.
                # Such windows must be rare and their two candidates equal to rounding; the oracle's
                # backward then routes through the GPU's winners, as it does through its rectifier signs.
                diff = np.flatnonzero(got.ravel() != am.ravel())
                assert diff.size <= max(2, got.size // 50000), ("max-pool winners", li, diff.size, got.size)
                planes = a.reshape(-1, a.shape[2] * a.shape[3])
                pl = diff // (am.shape[2] * am.shape[3])
                va, vb = planes[pl, got.ravel()[diff]], planes[pl, am.ravel()[diff]]
                assert np.all(np.abs(va - vb) <= 4e-6 * np.maximum(np.abs(vb), 1e-30)), ("max-pool winners", li)
                am = got.copy()
            else:
                assert np.array_equal(got, am), ("max-pool winners", li)
            aux_g.append(am)
        elif ly["kind"] == "softmax_ce":
            aux_g.append(orc32.softmax_ce(a.reshape(a.shape[0], -1), t["labels"])[1].reshape(a.shape))
        else:
            aux_g.append(None)
    return acts_g, aux_g


def _check_step(orc32, layers, in_shape, B, t, flags=0):
    gn = GpuNet(layers, in_shape, B, t)
    gn.step(SGD, flags)
    gn.sync()
    buckets = {k: v.copy() for k, v in t["buckets"].items()}
    loss, acts, aux = onet.forward(orc32, layers, t["x"], buckets, t["labels"], t["masks"])
    assert abs(float(host(gn.loss)[0]) - float(loss)) <= TOL * max(1.0, abs(float(loss)))
    for li in range(len(layers) - 1):
        if gn.fused(li):
            continue        # not materialised: the rectifier's output, checked at its own index, stands for it
        assert max_abs_rel(host(gn.act(li)), acts[li].ravel()) <= TOL, ("activation", li, layers[li]["kind"])
    acts_g, aux_g = _backward_state_from_gpu_forward(orc32, gn, layers, t, acts)
    grads, dact, _ = onet.backward(orc32, layers, t["x"], buckets, t["masks"], acts_g, aux_g)
    for li in grads:
        assert max_abs_rel(host(gn.g[li]), grads[li]) <= TOL, ("g_local", li)
        w, v = t["buckets"][li].copy(), np.zeros_like(t["buckets"][li])
        orc32.grad_reduce_sgd(w, v, host(gn.g[li]), t["peers"][li], *SGD)
        assert host(gn.w[li]).tobytes() == w.tobytes() and host(gn.v[li]).tobytes() == v.tobytes()
    return gn


def test_fully_connected_stack_at_b256(orc32):
    """fc6/fc7/fc8 of the AlexNet-shaped net (9216 -> 4096 -> 4096 -> 1000) with ReLU and dropout."""
    layers = [
        dict(kind="relu", inputs=[-1]),      # keeps an input gradient path alive for fc6's backward-data
        dict(kind="fc", inputs=[0], out=4096), dict(kind="relu", inputs=[1]), dict(kind="dropout", inputs=[2], p=0.5),
        dict(kind="fc", inputs=[3], out=4096), dict(kind="relu", inputs=[4]), dict(kind="dropout", inputs=[5], p=0.5),
        dict(kind="fc", inputs=[6], out=1000), dict(kind="softmax_ce", inputs=[7]),
    ]
    in_shape, B = (256, 6, 6), 256
    t = cg_synth.net_tensors(layers, in_shape, B, 2, seed=8, num_classes=1000)
    _check_step(orc32, layers, in_shape, B, t)


@pytest.mark.parametrize("B,K", [(16, 1), (64, 4), (256, 4)])
def test_whole_alexnet_shaped_iteration(orc32, B, K):
    """Configuration 4: B = 256 with K = 4 peers is the workload the benchmark's headline figure is
    quoted on (the oracle needs about half a minute for it), B = 64 the other per-worker batch the
    configuration names; B = 16 keeps the convolutions below the patch kernel's tile threshold, so
    both kernel families are checked inside a whole iteration."""
    layers, in_shape = cg_synth.alexnet_layers()
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=4, num_classes=1000)
    _check_step(orc32, layers, in_shape, B, t)


def test_inception_stack_at_its_real_shape(orc32):
    """Configuration 5: two inception modules on 192 x 28 x 28, B = 32, K = 8 peers."""
    layers, in_shape = cg_synth.inception_layers()
    B = 32
    t = cg_synth.net_tensors(layers, in_shape, B, 8, seed=5, num_classes=1000)
    _check_step(orc32, layers, in_shape, B, t)


def test_googlenet_shaped_iteration(orc32):
    """The paper's second benchmark net by shape (Table 1, GoogLeNet): stem and nine inception
    modules on 224 x 224 images, 58 parameter layers, here B = 4 with K = 2 peers, every
    activation, local gradient and updated bucket against the oracle."""
    layers, in_shape, _ = cg_synth.googlenet_layers()
    B = 4
    t = cg_synth.net_tensors(layers, in_shape, B, 2, seed=6, num_classes=1000)
    _check_step(orc32, layers, in_shape, B, t)


def test_update_of_the_eight_alexnet_buckets_in_one_launch(orc32):
    """Configuration 3 at its real sizes (60 965 224 parameters), K = 4: bit-exact, bucket by bucket."""
    sgd = (0.01, 0.9, 5e-4, 1.0)
    K = 4
    bk = cg_synth.sgd_buckets(K, seed=3, v_zero=False)
    for b in bk.values():
        b["g"], b["peers"] = b["g_local"], b["g_peers"]
    devs = {name: (dev(b["w"]), dev(b["v"]), dev(b["g"]), [dev(p) for p in b["peers"]]) for name, b in bk.items()}
    cg.cg_grad_reduce_sgd_multi([d[0] for d in devs.values()], [d[1] for d in devs.values()], [d[2] for d in devs.values()],
                                [d[3] for d in devs.values()], [b["w"].size for b in bk.values()], cg.cg_sgd(*sgd))
    for name, b in bk.items():
        orc32.grad_reduce_sgd(b["w"], b["v"], b["g"], b["peers"], *sgd)
        assert host(devs[name][0]).tobytes() == b["w"].tobytes(), name
        assert host(devs[name][1]).tobytes() == b["v"].tobytes(), name


def test_update_of_a_bucket_beyond_four_gibibytes(orc32):
    """n = 2^30 + 2^20 + 3 parameters: every buffer is larger than 4 GiB, so element and byte offsets
    leave 32 bits; K = 1, bit-exact against the oracle over the whole range.  Inputs are drawn on the
    GPU (seeded) and copied to the host for the oracle."""
    n = (1 << 30) + (1 << 20) + 3
    sgd = (0.01, 0.9, 5e-4, 1.0)
    gen = torch.Generator(device="cuda").manual_seed(33)
    dw = torch.empty(n, device="cuda").normal_(0.0, 1e-2, generator=gen)
    dv = torch.empty(n, device="cuda").normal_(0.0, 1e-4, generator=gen)
    dg = torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=gen)
    dp = torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=gen)
    w, v, g, p = (t.cpu().numpy() for t in (dw, dv, dg, dp))
    cg.cg_grad_reduce_sgd(dw, dv, dg, [dp], n, cg.cg_sgd(*sgd))
    orc32.grad_reduce_sgd(w, v, g, [p], *sgd)
    gw, gv = dw.cpu().numpy(), dv.cpu().numpy()
    for got, ref, name in ((gw, w, "w"), (gv, v, "v")):
        bad = np.flatnonzero(got.view(np.uint32) != ref.view(np.uint32))
        assert bad.size == 0, (name, bad[:5], bad.size)
    assert np.array_equal(dg.cpu().numpy().view(np.uint32), g.view(np.uint32))       # inputs untouched


def _sample_fwd(x, w, b, c, n, m, oh, ow):
    """One output element from the definition, in double."""
    G = c["groups"]; Cg = c["C"] // G; Mg = c["M"] // G; g = m // Mg
    acc = float(b[m])
    for ci in range(Cg):
        for kh in range(c["k"]):
            ih = oh * c["stride"] - c["pad"] + kh
            if not 0 <= ih < c["H"]:
                continue
            for kw in range(c["k"]):
                iw = ow * c["stride"] - c["pad"] + kw
                if 0 <= iw < c["H"]:
                    acc += float(x[n, g * Cg + ci, ih, iw]) * float(w[m, ci, kh, kw])
    return acc


def _dot64(a, b):
    """<a, b> accumulated in double, one slice of the leading axis at a time."""
    return float(sum(np.dot(a[i].ravel().astype(np.float64), b[i].ravel().astype(np.float64)) for i in range(a.shape[0])))


def _check_layer_by_samples_and_adjoints(c, x, w, b, dy, B, n_samples=40):
    d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    dx_, dw_, db_, dy_ = dev(x), dev(w), dev(b), dev(dy)
    y = host(conv_fwd(d, dx_, dw_, db_))
    assert np.isfinite(y).all()
    rng = np.random.default_rng(0)
    OH = y.shape[2]
    scale = np.abs(y).max()
    picks = [(0, 0, 0, 0), (B - 1, c["M"] - 1, OH - 1, OH - 1)] + \
        [tuple(int(rng.integers(0, hi)) for hi in (B, c["M"], OH, OH)) for _ in range(n_samples)]
    for (n, m, oh, ow) in picks:
        ref = _sample_fwd(x, w, b, c, n, m, oh, ow)
        assert abs(float(y[n, m, oh, ow]) - ref) <= TOL * scale, (n, m, oh, ow)
    # adjoint identities in double on the host: <conv(x,w), dy> = <x, bwd_data(dy,w)> = <w, bwd_weight(x,dy)>
    y0 = y - b.reshape(1, -1, 1, 1)
    lhs = _dot64(y0, dy)
    dxg = host(conv_bwd_data(d, dy_, dw_))
    gdw, gdb = conv_bwd_weight(d, dx_, dy_)
    gdw, gdb = host(gdw), host(gdb)
    norm = float(np.sqrt(_dot64(y0, y0)) * np.sqrt(_dot64(dy, dy)))
    assert abs(lhs - _dot64(dxg, x)) <= 1e-4 * norm
    assert abs(lhs - _dot64(gdw, w)) <= 1e-4 * norm
    rdb = dy.sum(axis=(0, 2, 3), dtype=np.float64)
    assert max_abs_rel(gdb, rdb) <= TOL
    # sampled backward-weight elements straight from the definition
    Cg = c["C"] // c["groups"]; Mg = c["M"] // c["groups"]
    s, p = c["stride"], c["pad"]
    wscale = np.abs(gdw).max()
    for _ in range(6):
        m, ci, kh, kw = (int(rng.integers(0, hi)) for hi in (c["M"], Cg, c["k"], c["k"]))
        g = m // Mg
        oh_lo, oh_hi = max(0, -(-(p - kh) // s)), min(OH - 1, (c["H"] - 1 + p - kh) // s)
        ow_lo, ow_hi = max(0, -(-(p - kw) // s)), min(OH - 1, (c["H"] - 1 + p - kw) // s)
        xs = x[:, g * Cg + ci, oh_lo * s - p + kh:oh_hi * s - p + kh + 1:s, ow_lo * s - p + kw:ow_hi * s - p + kw + 1:s]
        ref = float((xs.astype(np.float64) * dy[:, m, oh_lo:oh_hi + 1, ow_lo:ow_hi + 1]).sum())
        assert abs(float(gdw[m, ci, kh, kw]) - ref) <= TOL * wscale, (m, ci, kh, kw)
    # sampled backward-data elements straight from the definition (stride 1 only)
    if s == 1:
        xscale = np.abs(dxg).max()
        for _ in range(6):
            n, ch, ih, iw = (int(rng.integers(0, hi)) for hi in (B, c["C"], c["H"], c["H"]))
            g = ch // Cg
            ref = 0.0
            for kh in range(c["k"]):
                for kw in range(c["k"]):
                    oh, ow = ih + p - kh, iw + p - kw
                    if 0 <= oh < OH and 0 <= ow < OH:
                        ref += float(np.dot(dy[n, g * Mg:(g + 1) * Mg, oh, ow].astype(np.float64),
                                            w[g * Mg:(g + 1) * Mg, ch - g * Cg, kh, kw].astype(np.float64)))
            assert abs(float(dxg[n, ch, ih, iw]) - ref) <= TOL * xscale, (n, ch, ih, iw)


@pytest.mark.parametrize("layer", list(cg_synth.ALEXNET_CONVS))
def test_alexnet_conv_layer_at_b256_samples_and_adjoints(layer):
    B = 256
    c, x, w, b, dy = cg_synth.conv_layer_tensors(layer, B, seed=1 + list(cg_synth.ALEXNET_CONVS).index(layer))
    _check_layer_by_samples_and_adjoints(c, x, w, b, dy, B)


def test_conv_near_the_two_gibibyte_tensor_limit():
    """The library takes tensors of fewer than 2^29 elements (byte offsets fit 31 bits).  4096 images of
    160 x 27 x 27 are 477 757 440 elements, 89 % of that: the offsets of the last images use the top of
    the range in all three passes (5x5 window, padding 2: the kernels that stage raw image rows)."""
    B = 4096
    cfg = dict(C=160, H=27, M=16, k=5, stride=1, pad=2, groups=1)
    c, x, w, b, dy = cg_synth.conv_layer_tensors("near_limit", B, seed=29, cfg=cfg)
    assert x.size < (1 << 29) and x.size > 0.85 * (1 << 29)
    _check_layer_by_samples_and_adjoints(c, x, w, b, dy, B, n_samples=24)
