"""Seeded synthetic inputs for the SharePrefill hot path.

This package only *produces inputs* (Q/K/V bit patterns, the head-to-cluster map
and the pivotal-head list).  It holds none of the method's arithmetic: no
attention, no block scores, no mask selection.  Both the CPU oracle's tests and
the HIP path's tests/bench draw their inputs from here so that the two sides see
identical bf16 bits.
"""
from .generator import (LayerConfig, CONFIGS, make_layer, bf16_bits_to_f32,
                        f32_to_bf16_bits, random_qkv)

__all__ = ["LayerConfig", "CONFIGS", "make_layer", "bf16_bits_to_f32",
           "f32_to_bf16_bits", "random_qkv"]
