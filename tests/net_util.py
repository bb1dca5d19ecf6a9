"""Drive cg_train_step from the plain-dict layer lists (device memory via torch only)."""
import numpy as np
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import dev


class GpuNet:
    def __init__(self, layers, in_shape, B, tensors):
        self.layers, self.B = layers, B
        self.net = cg.Net(layers, B, in_shape)
        self.x, self.labels = dev(tensors["x"]), dev(tensors["labels"])
        self.w, self.v, self.g, self.peers = {}, {}, {}, {}
        for li, bucket in tensors["buckets"].items():
            assert cg.cg_net_param_count(self.net, li) == bucket.size
            self.w[li] = dev(bucket)
            self.v[li] = torch.zeros_like(self.w[li])
            self.g[li] = torch.full_like(self.w[li], float("nan"))
            self.peers[li] = [dev(p) for p in tensors["peers"][li]]
            cg.cg_net_bind(self.net, li, self.w[li], self.v[li], self.g[li], self.peers[li])
        self.masks = {li: dev(m) for li, m in tensors["masks"].items()}
        self.ws = torch.empty(cg.cg_net_workspace_bytes(self.net), dtype=torch.uint8, device="cuda")
        self.loss = torch.zeros(4, device="cuda")
        self.s0, self.s1 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()

    def step(self, sgd, flags=0):
        cg.cg_train_step(self.net, self.x, self.labels, self.masks, cg.cg_sgd(*sgd), self.ws, self.s0, self.s1,
                         self.loss, flags)

    def sync(self):
        self.s0.synchronize(); self.s1.synchronize(); torch.cuda.synchronize()

    def fused(self, layer):
        """True if this layer's own output is not materialised (the rectifier that follows is folded
        into its store; its buffer then holds the rectifier's output)."""
        return bool(cg.cg_net_layer_fused(self.net, layer) & 1)

    def grad_folded(self, layer):
        """True if the gradient with respect to this layer's output is not materialised (a rectifier
        whose backward is folded into its consumer's backward kernel)."""
        return bool(cg.cg_net_layer_fused(self.net, layer) & 2)

    def act(self, layer, which=0):
        return cg.cg_net_tensor(self.net, layer, which, self.ws)
