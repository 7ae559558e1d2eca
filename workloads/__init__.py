"""Seeded synthetic inputs for the integer-only inference path.

This package is the only code shared by the CPU oracle's tests and the HIP
library's tests/benchmark.  It draws random integer tensors (activations,
weights, biases, dyadic multipliers and shifts) with the shapes and value
ranges of the paper's ResNet18 / ResNet50 workloads and lays them out in the
byte formats the C interface documents.  It contains none of the method's
arithmetic: no convolution, no requantisation, no pooling.
"""
from .layers import resnet_layers, resnet_group_names  # noqa: F401
from .gen import (  # noqa: F401
    pack_nibbles,
    conv_case,
    int4_sweep_shapes,
    make_resnet,
    make_image_batch,
    draw_bits,
)
