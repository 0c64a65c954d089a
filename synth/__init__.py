"""Seeded synthetic MoE-layer inputs shared by the CPU oracle tests and the HIP path.

This package manufactures inputs only (activations, router logits, RTN-quantised expert
weights, low-rank factors).  It contains none of the forward-pass arithmetic: no dequantisation,
no projection, no routing, no packing.
"""
from .inputs import (CONFIGS, LayerConfig, Layer, make_layer, make_x, make_logits,
                     bf16_round, bf16_bits_to_f32, f32_to_bf16_bits, rtn_quantize, make_lotile, lotile_grid, make_lotile_fp8, fp8_e4m3_encode,
                     SharedLayer, make_shared_layer, make_planted_experts, tile_matrix,
                     Fp8Layer, make_layer_fp8)

__all__ = ["CONFIGS", "LayerConfig", "Layer", "make_layer", "make_x", "make_logits",
           "bf16_round", "bf16_bits_to_f32", "f32_to_bf16_bits", "rtn_quantize", "make_lotile", "lotile_grid", "make_lotile_fp8", "fp8_e4m3_encode",
           "SharedLayer", "make_shared_layer", "make_planted_experts", "tile_matrix",
           "Fp8Layer", "make_layer_fp8"]
