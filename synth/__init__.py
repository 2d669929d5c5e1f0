"""Seeded synthetic inputs: layer graphs, folded weights, images and schemes.

This package only *produces inputs* (shapes, random tensors, scheme tables).
It contains none of the scored method's arithmetic (no quantizer, no
convolution, no arithmetic-intensity formula) and imports neither the CPU
oracle nor the HIP library; both of those consume what it returns as plain
numpy arrays.
"""
from .graphs import (  # noqa: F401
    DESC_FIELDS, KIND_CONV, KIND_DEPTHWISE, KIND_FC, ACT_NONE, ACT_RELU, ACT_RELU6,
    resnet_cifar, mobilenetv2_32, plain_convnet20, heavy_early_resnet20,
    desc_array, n_scheme_layers,
)
from .data import make_model, make_images, make_workload, BITS_ALPHABET  # noqa: F401
