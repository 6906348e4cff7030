"""Seeded synthetic inputs for PCONV sparse 3x3 convolution layers.

This module only *draws* data: weights, pattern ids, connectivity masks, pattern
tables, biases and activations with the shapes and sparsity structure of the
workloads the paper evaluates (VGG-16 / ResNet-50 3x3 layers, pattern pruning
2.25x plus connectivity pruning; Tables 1-2 and the "Experimental Results"
section).  It contains none of the method's arithmetic (no masking, no packing,
no convolution) and is the only code shared by the CPU oracle's tests and the
HIP path's tests.
"""
from .gen import (  # noqa: F401
    PATTERN_TABLE, DENSE_MASK, LayerSpec, config_layers, make_layer, make_input,
    vgg16_conv_shapes, resnet50_conv3x3_shapes, base_seed, to_bf16_values,
    nnz_of_layer,
)
