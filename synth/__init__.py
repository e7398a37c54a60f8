"""Seeded synthetic inputs and network specifications.

This module serves both the CPU oracle and the HIP path.  It holds no part of
the method's arithmetic: only a counter-based random generator, the layer
records that describe a network, and the recipe for weights / images / labels.
"""
from .rng import splitmix64, uniform01, normal, labels_uniform
from .netspec import (
    CONV, BN, RELU, ADD, MAXPOOL, GAP, FC, SOFTMAX_CE, BIAS, KIND_NAMES,
    Layer, NetSpec, bottleneck_unit, vgg, vgg16, resnet, resnet18, resnet34, resnet50, resnet101, resnet152,
    param_count, init_params, make_batch,
)

__all__ = [
    "splitmix64", "uniform01", "normal", "labels_uniform",
    "CONV", "BN", "RELU", "ADD", "MAXPOOL", "GAP", "FC", "SOFTMAX_CE", "BIAS", "KIND_NAMES",
    "Layer", "NetSpec", "bottleneck_unit", "vgg", "vgg16", "resnet", "resnet18", "resnet34", "resnet50", "resnet101",
    "resnet152", "param_count", "init_params", "make_batch",
]
