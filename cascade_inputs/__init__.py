"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This module holds no arithmetic of the method: it names the five workload
configurations, draws random tensors of their shapes, draws token-to-shard
assignments, and rounds values onto the bf16 grid so that both sides consume
bit-identical inputs.  Neither the oracle nor the HIP library imports the other;
both may import this.
"""
from .configs import CONFIGS, LayerConfig, get_config
from .generate import (make_assignment, make_hidden, make_layer_weights, make_head_weights,
                       round_to_bf16, bf16_bits, bf16_bits_to_f32, config_seed)

__all__ = ["CONFIGS", "LayerConfig", "get_config", "make_assignment", "make_hidden",
           "make_layer_weights", "make_head_weights", "round_to_bf16", "bf16_bits", "bf16_bits_to_f32",
           "config_seed"]
