"""Seeded synthetic inputs for the CARD verify step (weights, tokens, candidates).

This module holds no arithmetic of the method itself: it only produces the
numbers that both the CPU oracle and the HIP path consume.  Every value is a
pure function of (seed, tensor tag, layer, flat index) computed with integer
operations only, so the same tensor comes out bit-identical on any torch
device (CPU here, the GPU on the measurement box).
"""
from .configs import ModelShape, SHAPES, shape_by_name
from .generate import (
    TENSOR_TAGS,
    bf16_matrix,
    gains,
    uniform_tokens,
    layer_matrices,
    stream_key,
    plant_candidates,
)

__all__ = [
    "ModelShape",
    "SHAPES",
    "shape_by_name",
    "TENSOR_TAGS",
    "bf16_matrix",
    "gains",
    "uniform_tokens",
    "layer_matrices",
    "stream_key",
    "plant_candidates",
]
