"""Seeded synthetic inputs for the pair-search path (weights, channel norms, raw normal draws).

This module serves both the CPU oracle and the HIP path and therefore contains none of the
method's arithmetic: only random draws with the shapes and value structure of LLM linear layers
(heavy-tailed Student-t entries, log-normal per-row scales, sparse outliers, log-normal channel
norms) and the bf16 <-> fp32 container conversions.  Nothing here comes from a dataset or a
model checkpoint; the paper's own measurements use real model weights and calibration text,
which these inputs stand in for.
"""
from .generate import (  # noqa: F401
    bf16_round, bf16_bits, bf16_bits_to_f32, student_t_weights, channel_norms,
    normal_draws, CONFIGS, make_config, layer_shapes_7b, model_7b_layers, model_7b_layer,
)
