"""Seeded synthetic inputs for the OWQ mixed-precision linear layer.

This module only draws random tensors and arranges them in the plain
(unpacked) description of a layer.  It holds none of the method's arithmetic:
no packing, no dequantisation, no matrix product.  Both the CPU oracle's tests
and the GPU library's tests and bench take their inputs from here.
"""
from .layers import LayerSpec, Layer, make_layer, make_weights, make_x, CONFIGS, config_layers

__all__ = ["LayerSpec", "Layer", "make_layer", "make_weights", "make_x", "CONFIGS", "config_layers"]
