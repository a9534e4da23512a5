"""Seeded synthetic workloads: configuration records and input generators.

This module holds no arithmetic of the training method.  It only names the
problem sizes and draws the random tensors (weights, activations, upstream
gradients, token ids, Adam moments) that both the CPU oracle and the HIP path
consume, so that the two sides see byte-identical inputs without sharing any
code of the method itself.
"""
from .configs import CONFIGS, LayerConfig, get_config, shard_of  # noqa: F401
from .generate import (  # noqa: F401
    draw_layer_params,
    draw_activations,
    draw_adam_state,
    draw_token_ids,
    draw_stack_params,
)
