"""Seeded synthetic inputs for the MoE-layer share and for the host planners.

This package holds only input recipes (shapes, seeds, value distributions, the
skewed traffic-matrix recipe).  It contains none of the method's arithmetic:
no gating, no permutation, no FFN, no scheduling.  Both the CPU oracle's tests
and the GPU library's tests draw their inputs from here so that the two sides
see the same host arrays.
"""
from .configs import LayerConfig, CONFIGS, get_config, scaled
from .generate import (to_bf16_grid, round_to_dtype, make_layer_inputs, make_expert_weights,
                       zipf_popularity, make_traffic_matrix, make_link_rates, rng_for)

__all__ = ["LayerConfig", "CONFIGS", "get_config", "scaled", "to_bf16_grid", "round_to_dtype",
           "make_layer_inputs", "make_expert_weights", "zipf_popularity", "make_traffic_matrix",
           "make_link_rates", "rng_for"]
