"""Layer lists and seeded tensors for the five benchmark configurations."""
import math

import numpy as np

# --- configuration 2: the five AlexNet-shaped convolution layers -------------------------
# (C, H, M, k, stride, pad, groups); input is square HxH.
ALEXNET_CONVS = {
    "conv1": dict(C=3, H=227, M=96, k=11, stride=4, pad=0, groups=1),
    "conv2": dict(C=96, H=27, M=256, k=5, stride=1, pad=2, groups=2),
    "conv3": dict(C=256, H=13, M=384, k=3, stride=1, pad=1, groups=1),
    "conv4": dict(C=384, H=13, M=384, k=3, stride=1, pad=1, groups=2),
    "conv5": dict(C=384, H=13, M=256, k=3, stride=1, pad=1, groups=2),
}

# --- configuration 3: parameter buckets (weights + bias per layer) -----------------------
ALEXNET_BUCKETS = {
    "conv1": 96 * 3 * 11 * 11 + 96,
    "conv2": 256 * 48 * 5 * 5 + 256,
    "conv3": 384 * 256 * 3 * 3 + 384,
    "conv4": 384 * 192 * 3 * 3 + 384,
    "conv5": 256 * 192 * 3 * 3 + 256,
    "fc6": 4096 * 9216 + 4096,
    "fc7": 4096 * 4096 + 4096,
    "fc8": 1000 * 4096 + 1000,
}


def _conv(src, M, k, stride=1, pad=0, groups=1):
    return dict(kind="conv", inputs=[src], M=M, k=k, stride=stride, pad=pad, groups=groups)


def _relu(src):
    return dict(kind="relu", inputs=[src])


def _lrn(src):
    return dict(kind="lrn", inputs=[src], size=5, alpha=1e-4, beta=0.75, kappa=1.0)


def _maxpool(src, k, stride, pad=0):
    return dict(kind="maxpool", inputs=[src], k=k, stride=stride, pad=pad)


def tiny_cnn_layers():
    """Configuration 1: conv 3->16 k3 p1, ReLU, conv 16->32 k3 p1, ReLU, global average
    pool, FC 32->10, softmax cross-entropy.  Input 8x3x32x32."""
    L = [
        _conv(-1, 16, 3, pad=1), _relu(0),
        _conv(1, 32, 3, pad=1), _relu(2),
        dict(kind="avgpool", inputs=[3]),
        dict(kind="fc", inputs=[4], out=10),
        dict(kind="softmax_ce", inputs=[5]),
    ]
    return L, (3, 32, 32)


def alexnet_layers(num_classes=1000):
    """Configuration 4: five convolutions with ReLU, LRN after conv1/conv2, 3x3 stride-2
    max-pool after conv1, conv2, conv5, then FC 9216->4096->4096->classes with ReLU and
    dropout 0.5, softmax cross-entropy.  Input 3x227x227."""
    L = []

    def add(layer):
        L.append(layer)
        return len(L) - 1

    t = add(_conv(-1, 96, 11, stride=4))
    t = add(_relu(t)); t = add(_lrn(t)); t = add(_maxpool(t, 3, 2))
    t = add(_conv(t, 256, 5, pad=2, groups=2))
    t = add(_relu(t)); t = add(_lrn(t)); t = add(_maxpool(t, 3, 2))
    t = add(_conv(t, 384, 3, pad=1)); t = add(_relu(t))
    t = add(_conv(t, 384, 3, pad=1, groups=2)); t = add(_relu(t))
    t = add(_conv(t, 256, 3, pad=1, groups=2)); t = add(_relu(t))
    t = add(_maxpool(t, 3, 2))
    t = add(dict(kind="fc", inputs=[t], out=4096)); t = add(_relu(t))
    t = add(dict(kind="dropout", inputs=[t], p=0.5))
    t = add(dict(kind="fc", inputs=[t], out=4096)); t = add(_relu(t))
    t = add(dict(kind="dropout", inputs=[t], p=0.5))
    t = add(dict(kind="fc", inputs=[t], out=num_classes))
    add(dict(kind="softmax_ce", inputs=[t]))
    return L, (3, 227, 227)


def inception_layers(modules=2, cin=192, hw=28, num_classes=1000):
    """Configuration 5: `modules` inception blocks on cin x hw x hw.  Branches: 1x1/64;
    1x1/96 -> 3x3/128; 1x1/16 -> 5x5/32; 3x3 s1 p1 max-pool -> 1x1/32; every convolution
    followed by ReLU; channel concat (256 out).  Then global average pool, FC, softmax CE."""
    L = []

    def add(layer):
        L.append(layer)
        return len(L) - 1

    src = -1
    for _ in range(modules):
        b1 = add(_relu(add(_conv(src, 64, 1))))
        b2 = add(_relu(add(_conv(src, 96, 1))))
        b2 = add(_relu(add(_conv(b2, 128, 3, pad=1))))
        b3 = add(_relu(add(_conv(src, 16, 1))))
        b3 = add(_relu(add(_conv(b3, 32, 5, pad=2))))
        b4 = add(_maxpool(src, 3, 1, 1))
        b4 = add(_relu(add(_conv(b4, 32, 1))))
        src = add(dict(kind="concat", inputs=[b1, b2, b3, b4]))
    t = add(dict(kind="avgpool", inputs=[src]))
    t = add(dict(kind="fc", inputs=[t], out=num_classes))
    add(dict(kind="softmax_ce", inputs=[t]))
    return L, (cin, hw, hw)


# (1x1, 3x3 reduce, 3x3, 5x5 reduce, 5x5, pool projection) of the nine modules of the 22-layer
# inception network (Szegedy et al., "Going deeper with convolutions", 2014, Table 1)
_INCEPTION_V1_MODULES = [
    ("3a", 64, 96, 128, 16, 32, 32), ("3b", 128, 128, 192, 32, 96, 64), "pool",
    ("4a", 192, 96, 208, 16, 48, 64), ("4b", 160, 112, 224, 24, 64, 64), ("4c", 128, 128, 256, 24, 64, 64),
    ("4d", 112, 144, 288, 32, 64, 64), ("4e", 256, 160, 320, 32, 128, 128), "pool",
    ("5a", 256, 160, 320, 32, 128, 128), ("5b", 384, 192, 384, 48, 128, 128),
]


def googlenet_layers(num_classes=1000, hw=224):
    """The paper's second benchmark net (Table 1, GoogLeNet, batch 32) by shape: stem (7x7/2 conv,
    pool, LRN, 1x1 and 3x3 conv, LRN, pool), nine inception modules with two stride-2 pools
    between them, global average pool, dropout 0.4, FC, softmax cross-entropy.  Every
    convolution is followed by ReLU; pools are 3x3 (stride 2 between stages, stride 1 pad 1
    inside a module).  The two auxiliary classifiers of the training net are left out.
    Returns (layers, input shape, names) with names[i] the label of parameter layer i."""
    L, names = [], {}

    def add(layer, name=None):
        L.append(layer)
        if name:
            names[len(L) - 1] = name
        return len(L) - 1

    def conv(src, M, k, name, stride=1, pad=0):
        return add(_relu(add(_conv(src, M, k, stride=stride, pad=pad), name)))

    t = conv(-1, 64, 7, "conv1", stride=2, pad=3)
    t = add(_maxpool(t, 3, 2)); t = add(_lrn(t))
    t = conv(t, 64, 1, "conv2_reduce")
    t = conv(t, 192, 3, "conv2", pad=1)
    t = add(_lrn(t)); t = add(_maxpool(t, 3, 2))
    for m in _INCEPTION_V1_MODULES:
        if m == "pool":
            t = add(_maxpool(t, 3, 2))
            continue
        tag, c1, r3, c3, r5, c5, pp = m
        b1 = conv(t, c1, 1, tag + "_1x1")
        b2 = conv(conv(t, r3, 1, tag + "_3x3_reduce"), c3, 3, tag + "_3x3", pad=1)
        b3 = conv(conv(t, r5, 1, tag + "_5x5_reduce"), c5, 5, tag + "_5x5", pad=2)
        b4 = conv(add(_maxpool(t, 3, 1, 1)), pp, 1, tag + "_pool_proj")
        t = add(dict(kind="concat", inputs=[b1, b2, b3, b4]))
    t = add(dict(kind="avgpool", inputs=[t]))
    t = add(dict(kind="dropout", inputs=[t], p=0.4))
    t = add(dict(kind="fc", inputs=[t], out=num_classes), "classifier")
    add(dict(kind="softmax_ce", inputs=[t]))
    return L, (3, hw, hw), names


def _pool_out(H, k, s, p):
    o = -(-(H + 2 * p - k) // s) + 1
    if (o - 1) * s >= H + p:
        o -= 1
    return o


def infer_shapes(layers, in_shape):
    """Per-layer output shape (C, H, W); FC / avgpool / loss outputs are (C, 1, 1)."""
    shapes = []

    def src_shape(i):
        return in_shape if i < 0 else shapes[i]

    for ly in layers:
        C, H, W = src_shape(ly["inputs"][0])
        kind = ly["kind"]
        if kind == "conv":
            k, s, p = ly["k"], ly["stride"], ly["pad"]
            shapes.append((ly["M"], (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1))
        elif kind == "maxpool":
            shapes.append((C, _pool_out(H, ly["k"], ly["stride"], ly["pad"]),
                           _pool_out(W, ly["k"], ly["stride"], ly["pad"])))
        elif kind == "avgpool":
            shapes.append((C, 1, 1))
        elif kind == "fc":
            shapes.append((ly["out"], 1, 1))
        elif kind == "concat":
            shapes.append((sum(src_shape(i)[0] for i in ly["inputs"]), H, W))
        elif kind == "softmax_ce":
            shapes.append((1, 1, 1))
        else:  # relu, lrn, dropout
            shapes.append((C, H, W))
    return shapes


def param_layers(layers, in_shape):
    """[(layer index, weight shape, bias length)] for every conv / fc layer, in net order."""
    shapes = infer_shapes(layers, in_shape)
    out = []
    for i, ly in enumerate(layers):
        src = ly["inputs"][0]
        C, H, W = in_shape if src < 0 else shapes[src]
        if ly["kind"] == "conv":
            out.append((i, (ly["M"], C // ly["groups"], ly["k"], ly["k"]), ly["M"]))
        elif ly["kind"] == "fc":
            out.append((i, (ly["out"], C * H * W), ly["out"]))
    return out


def xavier_uniform(rng, shape):
    """U(-a, a), a = sqrt(6 / (fan_in + fan_out)); fan = channels * receptive field."""
    rf = int(np.prod(shape[2:])) if len(shape) > 2 else 1
    a = math.sqrt(6.0 / (shape[1] * rf + shape[0] * rf))
    return rng.uniform(-a, a, size=shape).astype(np.float32)


def conv_layer_tensors(name, B, seed, cfg=None):
    """Configuration 2 tensors for one layer: x, w ~ N(0,1)/sqrt(fan_in), bias ~ N(0,1)*0.1,
    dy ~ N(0,1)/sqrt(fan_out).  Returns (cfg, x, w, bias, dy)."""
    c = dict(cfg or ALEXNET_CONVS[name])
    rng = np.random.default_rng(seed)
    Cg = c["C"] // c["groups"]
    W_ = c.get("W", c["H"])
    fan_in = Cg * c["k"] * c["k"]
    fan_out = (c["M"] // c["groups"]) * c["k"] * c["k"]
    OH = (c["H"] + 2 * c["pad"] - c["k"]) // c["stride"] + 1
    OW = (W_ + 2 * c["pad"] - c["k"]) // c["stride"] + 1
    x = (rng.standard_normal((B, c["C"], c["H"], W_), dtype=np.float32) / np.float32(math.sqrt(fan_in)))
    w = (rng.standard_normal((c["M"], Cg, c["k"], c["k"]), dtype=np.float32) / np.float32(math.sqrt(fan_in)))
    bias = rng.standard_normal(c["M"], dtype=np.float32) * np.float32(0.1)
    dy = (rng.standard_normal((B, c["M"], OH, OW), dtype=np.float32) / np.float32(math.sqrt(fan_out)))
    return c, x, w, bias, dy


def conv_layer_int_tensors(cfg, B, seed, lim=3):
    """Small-integer tensors for one convolution layer: x, w, bias, dy uniform on the integers
    -lim..lim, stored as float32.  Every product and every partial sum of up to 2^24 / lim^2 terms is
    then an integer that fp32 represents exactly, so any summation order gives the same bits.
    Returns (cfg, x, w, bias, dy)."""
    c = dict(cfg)
    rng = np.random.default_rng(seed)
    Cg = c["C"] // c["groups"]
    W_ = c.get("W", c["H"])
    OH = (c["H"] + 2 * c["pad"] - c["k"]) // c["stride"] + 1
    OW = (W_ + 2 * c["pad"] - c["k"]) // c["stride"] + 1

    def draw(shape):
        return rng.integers(-lim, lim + 1, size=shape).astype(np.float32)

    return (c, draw((B, c["C"], c["H"], W_)), draw((c["M"], Cg, c["k"], c["k"])), draw((c["M"],)),
            draw((B, c["M"], OH, OW)))


def net_tensors(layers, in_shape, B, K, seed, num_classes, init="fan_in", peer_std=1e-3, bias_std=0.1):
    """Inputs of one training iteration: x ~ N(0,1), labels uniform, one parameter bucket
    (weights then bias, contiguous) per conv/fc layer, zero history, K peer gradient
    buckets ~ N(0, peer_std) per layer, Bernoulli(1-p) keep masks for dropout layers.
    Biases ~ N(0, bias_std): a model in the middle of training has non-zero biases, and with zeros the
    per-row and per-column bias paths of the kernels would add nothing that a test could see."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B,) + tuple(in_shape), dtype=np.float32)
    labels = rng.integers(0, num_classes, size=B).astype(np.int32)
    shapes = infer_shapes(layers, in_shape)
    buckets, peers, masks = {}, {}, {}
    for li, wshape, nb in param_layers(layers, in_shape):
        if init == "xavier":
            w = xavier_uniform(rng, wshape)
        else:
            fan_in = int(np.prod(wshape[1:]))
            w = rng.standard_normal(wshape, dtype=np.float32) / np.float32(math.sqrt(fan_in))
        b = rng.standard_normal(nb, dtype=np.float32) * np.float32(bias_std)
        buckets[li] = np.concatenate([w.ravel(), b]).astype(np.float32)
        peers[li] = [(rng.standard_normal(buckets[li].size, dtype=np.float32) * np.float32(peer_std))
                     for _ in range(K)]
    for i, ly in enumerate(layers):
        if ly["kind"] == "dropout":
            C, H, W = shapes[i]
            masks[i] = (rng.random((B, C * H * W)) >= ly["p"]).astype(np.uint8)
    return dict(x=x, labels=labels, buckets=buckets, peers=peers, masks=masks)


def sgd_buckets(K, seed=3, sizes=None, w_std=1e-2, g_std=1e-3, v_zero=True):
    """Configuration 3: per bucket w ~ N(0, w_std), v (zero or ~N(0, 1e-4)), local gradient
    and K peer gradients ~ N(0, g_std)."""
    sizes = dict(sizes or ALEXNET_BUCKETS)
    rng = np.random.default_rng(seed)
    out = {}
    for name, n in sizes.items():
        w = rng.standard_normal(n, dtype=np.float32) * np.float32(w_std)
        v = np.zeros(n, np.float32) if v_zero else rng.standard_normal(n, dtype=np.float32) * np.float32(1e-4)
        g = rng.standard_normal(n, dtype=np.float32) * np.float32(g_std)
        peers = [rng.standard_normal(n, dtype=np.float32) * np.float32(g_std) for _ in range(K)]
        out[name] = dict(w=w, v=v, g_local=g, g_peers=peers)
    return out
