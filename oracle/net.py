"""CPU oracle (test infrastructure only): one worker's whole SGD iteration.

Follows Fig. 1 (mini-batch SGD: forward, backward, update) with the
data-parallel update of Eq. 1 applied layer by layer (section 3, "layer-wise
model update"): forward through layers 1..L, loss, backward through layers
L..1 producing this worker's gradient bucket per layer, then for every layer
the (K+1)-buffer sum and the solver update.  The oracle runs these strictly one
after the other; the overlap of section 2.3 changes when things run, never
what they compute.

Layer lists are plain dicts (see cg_synth.workloads); parameter buckets hold the
weights followed by the bias.
"""
import numpy as np

from .cgo import Oracle, conv_desc


def _src(acts, x, i):
    return x if i < 0 else acts[i]


def forward(orc, layers, x, buckets, labels, masks):
    """Returns (loss, acts, aux) -- every layer's output and what backward needs."""
    acts, aux = [], []
    loss = None
    for li, ly in enumerate(layers):
        kind = ly["kind"]
        a = _src(acts, x, ly["inputs"][0])
        if kind == "conv":
            N, C, H, W = a.shape
            d = conv_desc(N, C, H, W, ly["M"], ly["k"], ly["stride"], ly["pad"], ly["groups"])
            nw = ly["M"] * (C // ly["groups"]) * ly["k"] * ly["k"]
            w, b = buckets[li][:nw], buckets[li][nw:]
            acts.append(orc.conv_fwd(d, a, w, b)); aux.append(d)
        elif kind == "relu":
            acts.append(orc.relu_fwd(a)); aux.append(None)
        elif kind == "lrn":
            y, sc = orc.lrn_fwd(a, ly["size"], ly["alpha"], ly["beta"], ly["kappa"])
            acts.append(y); aux.append(sc)
        elif kind == "maxpool":
            y, am = orc.maxpool_fwd(a, ly["k"], ly["stride"], ly["pad"])
            acts.append(y); aux.append(am)
        elif kind == "avgpool":
            acts.append(orc.avgpool_fwd(a)); aux.append(None)
        elif kind == "fc":
            B = a.shape[0]
            a2 = a.reshape(B, -1)
            IN = a2.shape[1]
            W_, b = buckets[li][:ly["out"] * IN].reshape(ly["out"], IN), buckets[li][ly["out"] * IN:]
            acts.append(orc.fc_fwd(a2, W_, b).reshape(B, ly["out"], 1, 1)); aux.append(None)
        elif kind == "dropout":
            acts.append(orc.dropout(a, masks[li], ly["p"]).reshape(a.shape)); aux.append(None)
        elif kind == "concat":
            acts.append(np.concatenate([_src(acts, x, i) for i in ly["inputs"]], axis=1)); aux.append(None)
        elif kind == "softmax_ce":
            B = a.shape[0]
            loss, dz = orc.softmax_ce(a.reshape(B, -1), labels)
            acts.append(np.full((1,), loss, orc.dtype)); aux.append(dz.reshape(a.shape))
        else:
            raise ValueError(kind)
    return loss, acts, aux


def backward(orc, layers, x, buckets, masks, acts, aux, need_input_grad=False):
    """Returns ({layer: gradient bucket}, {layer: d loss / d output})."""
    dact = {}
    grads = {}
    dxin = None

    def push(i, g):
        nonlocal dxin
        if i < 0:
            dxin = g if dxin is None else dxin + g
        else:
            dact[i] = g if i not in dact else dact[i] + g

    for li in range(len(layers) - 1, -1, -1):
        ly = layers[li]
        kind = ly["kind"]
        s0 = ly["inputs"][0]
        a = _src(acts, x, s0)
        if kind == "softmax_ce":
            push(s0, aux[li]); continue
        dy = dact[li]
        if kind == "conv":
            d = aux[li]
            nw = ly["M"] * (d.C // ly["groups"]) * ly["k"] * ly["k"]
            dw, db = orc.conv_bwd_weight(d, a, dy)
            grads[li] = np.concatenate([dw.ravel(), db])
            if s0 >= 0 or need_input_grad:
                push(s0, orc.conv_bwd_data(d, dy, buckets[li][:nw]))
        elif kind == "relu":
            push(s0, orc.relu_bwd(a, dy))
        elif kind == "lrn":
            push(s0, orc.lrn_bwd(a, acts[li], aux[li], dy, ly["size"], ly["alpha"], ly["beta"]))
        elif kind == "maxpool":
            push(s0, orc.maxpool_bwd(a.shape, ly["k"], ly["stride"], ly["pad"], dy, aux[li]))
        elif kind == "avgpool":
            push(s0, orc.avgpool_bwd(a.shape, dy))
        elif kind == "fc":
            B = a.shape[0]
            a2 = a.reshape(B, -1)
            IN = a2.shape[1]
            dy2 = dy.reshape(B, -1)
            dW, db = orc.fc_bwd_weight(a2, dy2)
            grads[li] = np.concatenate([dW.ravel(), db])
            if s0 >= 0 or need_input_grad:
                W_ = buckets[li][:ly["out"] * IN].reshape(ly["out"], IN)
                push(s0, orc.fc_bwd_data(dy2, W_).reshape(a.shape))
        elif kind == "dropout":
            push(s0, orc.dropout(dy, masks[li], ly["p"]).reshape(a.shape))
        elif kind == "concat":
            off = 0
            for i in ly["inputs"]:
                c = _src(acts, x, i).shape[1]
                push(i, np.ascontiguousarray(dy[:, off:off + c])); off += c
        else:
            raise ValueError(kind)
    return grads, dact, dxin


def train_step(orc, layers, x, labels, buckets, hist, peers, masks, lr, mu, wd, grad_scale=1.0):
    """One iteration.  buckets/hist are updated in place; returns (loss, local gradients)."""
    loss, acts, aux = forward(orc, layers, x, buckets, labels, masks)
    grads, _, _ = backward(orc, layers, x, buckets, masks, acts, aux)
    for li in sorted(grads, reverse=True):
        orc.grad_reduce_sgd(buckets[li], hist[li], grads[li], peers[li], lr, mu, wd, grad_scale)
    return loss, grads


def loss_only(orc, layers, x, labels, buckets, masks):
    return forward(orc, layers, x, buckets, labels, masks)[0]


__all__ = ["Oracle", "forward", "backward", "train_step", "loss_only"]
