"""Seeded synthetic inputs for the LCD table-lookup linear layer.

This module only *draws inputs* (codebooks, indices, activations, smoothing scales) with
the shapes and value distributions of the benchmark configurations.  It holds none of the
method's arithmetic: it never dequantises a weight, never divides an activation by its
smoothing scale and never forms a product.  Both the CPU oracle's tests and the GPU
path's tests/bench draw from here so that they see identical arrays.
"""
from .configs import CONFIGS, LayerSpec, Config, get_config
from .generators import (
    centroid_set,
    make_codebook,
    make_indices,
    outlier_channels,
    make_activations,
    make_smoothing,
    make_layer,
    make_layer_uniform,
    seed_for,
)

__all__ = [
    "CONFIGS", "LayerSpec", "Config", "get_config", "centroid_set", "make_codebook",
    "make_indices", "outlier_channels", "make_activations", "make_smoothing",
    "make_layer", "make_layer_uniform", "seed_for",
]
