"""Seeded synthetic conv workloads (layer shapes and random tensors).

This package holds shapes and random-number recipes only: none of the
arithmetic of weight transformation or convolution lives here, so both the
CPU oracle's tests and the GPU library's tests may draw inputs from it.
"""
from .stacks import ConvLayer, stack, STACK_NAMES, table2_layer  # noqa: F401
from .gen import layer_tensors, BASE_SEED  # noqa: F401
