"""Seeded synthetic workloads shared by the CPU oracle's tests and the GPU path.

This module describes WHAT is run (layer lists, tensor shapes, value
distributions, seeds) and holds none of the method's arithmetic: no
convolution, no layer formula, no update rule.  Everything is numpy on the
host; callers hand the arrays bit-identically to whichever implementation
they drive.

The paper trains AlexNet (B=256) and GoogLeNet (B=32) on ImageNet (Table 1,
section 4).  Neither the dataset nor trained weights are used here: dense
convolution cost does not depend on the values, so N(0,1) tensors of the same
shapes stand in for the images.
"""
from .workloads import (  # noqa: F401
    ALEXNET_CONVS, ALEXNET_BUCKETS, alexnet_layers, tiny_cnn_layers, inception_layers, googlenet_layers,
    infer_shapes, param_layers, conv_layer_tensors, conv_layer_int_tensors, net_tensors, sgd_buckets, xavier_uniform,
)
