"""Seeded synthetic inputs for the vector-quantized linear layer.

This package serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It only *produces inputs* (random tables, random indices, the
bit-packed index streams, activations, column permutations, Hessians, weights); it holds none of the decode
arithmetic: no unpacker, no lookup, no dequantisation, no matmul.
"""
from .generators import splitmix64, uniform01, normal, to_fp16, random_indices, tensor_seed, permutation
from .pack import pack_indices, row_stride_bytes, index_bits
from .configs import VQLayer, make_layer, make_activations, make_hessian, make_weights, CONFIGS, config_layers

__all__ = [
    "splitmix64", "uniform01", "normal", "to_fp16", "random_indices", "tensor_seed", "permutation",
    "pack_indices", "row_stride_bytes", "index_bits",
    "VQLayer", "make_layer", "make_activations", "make_hessian", "make_weights", "CONFIGS", "config_layers",
]
