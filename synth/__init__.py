"""Seeded synthetic inputs (network descriptions, parameters, images).

This package holds data generation only: array shapes, random draws and the
wiring of the residual networks.  It contains none of the method's arithmetic
(no convolution, no batch-norm evaluation, no folding, no pruning) and is the
only code shared by the CPU oracle's tests and the GPU library's tests.
"""
from .resnets import (  # noqa: F401
    BASE_SEED,
    CONFIG_NAMES,
    make_config,
    make_block_model,
    make_cifar_resnet,
    make_imagenet_basic_resnet,
    make_imagenet_bottleneck_resnet,
    make_input,
    make_paper_workload,
    PAPER_WORKLOADS,
    prunable_convs,
)
