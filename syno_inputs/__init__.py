"""Shared synthetic inputs: operator descriptions (pGraphs) and seeded tensors.

Used by the tests, the benchmark, the CPU checker's wrapper and the GPU
binding.  Holds no operator arithmetic.
"""
from .descriptor import (BF16, EXPAND, F32, KIND_NAMES, MERGE, REDUCE, SHARE, SHIFT, SPLIT, STRIDE,
                         UNFOLD, Builder, OpDesc, Prim)
from .rng import Stream, bf16_bits_to_f32, to_bf16_bits
from . import workloads

__all__ = ["BF16", "F32", "SPLIT", "MERGE", "SHIFT", "EXPAND", "UNFOLD", "STRIDE", "REDUCE", "SHARE",
           "KIND_NAMES", "Builder", "OpDesc", "Prim", "Stream", "to_bf16_bits", "bf16_bits_to_f32",
           "workloads"]
