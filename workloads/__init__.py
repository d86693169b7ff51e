"""Synthetic workloads: network tables of the five benchmark configurations and seeded
input generators.

This module holds **no arithmetic of the method** (no convolution, pooling, loss, gradient
or update): only shapes, block/batch tables and random draws.  Both the CPU oracle tests
and the GPU tests/bench take their inputs from here, which is the only thing they share.

Tensors are produced in the logical layout of the paper's notation: NCHW activations,
OIHW convolution weights, [out][in] linear weights, int32 labels.
"""
from .configs import (Block, Config, LayerSpec, config, config_names, resnet_layers,  # noqa: F401
                      vgg_layers)
from .gen import gen_batch, gen_class_patterns, gen_layer_params, rng_for  # noqa: F401
