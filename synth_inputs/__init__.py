"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU harness.

This package only *draws data*: templates (field slots + dependency edges),
model dimensions, bf16-representable weight tensors, prefix embeddings and
start tokens.  It contains none of the method's arithmetic (no masks, no
ancestors, no attention, no normalisation); both sides derive those from the
data produced here with code of their own.
"""
from .configs import (ModelDims, Template, model_dims, template, workload_seed,
                      random_dag_template, chain_template, edgeless_template)
from .tensors import (bf16_round, bf16_bits, bits_to_f32, draw_weights,
                      draw_layer_weights, draw_prefix_embeddings,
                      draw_tokens, draw_normal_bf16, LAYER_KEYS)

__all__ = [
    "ModelDims", "Template", "model_dims", "template", "workload_seed",
    "random_dag_template", "chain_template", "edgeless_template",
    "bf16_round", "bf16_bits", "bits_to_f32", "draw_weights",
    "draw_layer_weights", "draw_prefix_embeddings", "draw_tokens",
    "draw_normal_bf16", "LAYER_KEYS",
]
