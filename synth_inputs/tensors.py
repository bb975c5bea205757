"""Seeded tensors: weights, prefix embeddings, tokens.

Every floating-point tensor drawn here is rounded once to a bf16-representable
value (round to nearest, ties to even), because the workloads hold weights,
embeddings and cached K/V in bf16.  The rounded values are *data*: the oracle
reads them as exact fp64 numbers, the GPU path uploads their 16-bit patterns.
"""
from __future__ import annotations

import numpy as np

from .configs import ModelDims, workload_seed

LAYER_KEYS = ("g1", "wqkv", "wo", "g2", "wgu", "wd")


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 numbers they denote."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is bf16-representable."""
    return bits_to_f32(bf16_bits(x))


def draw_normal_bf16(rng: np.random.Generator, shape, std: float = 1.0,
                     mean: float = 0.0, bits: bool = False) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return bf16_bits(x) if bits else bf16_round(x)


def _layer_shapes(d: ModelDims):
    return {
        "g1": (d.d_model,),
        "wqkv": (d.qkv_out, d.d_model),                 # rows: Q heads, K heads, V heads
        "wo": (d.d_model, d.n_q_heads * d.head_dim),
        "g2": (d.d_model,),
        "wgu": (2 * d.d_mlp, d.d_model),                # rows: gate then up
        "wd": (d.d_model, d.d_mlp),
    }


def draw_layer_weights(cfg_id: int, d: ModelDims, layer: int, *, random_gains: bool,
                       bits: bool = False, std: float = 0.02) -> dict:
    """One decoder layer.  Every matrix is [out_features][in_features], so a
    projection is y = x @ W.T.  `bits=True` returns uint16 bf16 patterns for
    the matrices (gains are always fp32 arrays of bf16-representable values)."""
    rng = workload_seed(cfg_id, "weights", 1 + layer)
    out = {}
    for k, shp in _layer_shapes(d).items():
        if k in ("g1", "g2"):
            out[k] = (draw_normal_bf16(rng, shp, std, 1.0) if random_gains
                      else np.ones(shp, dtype=np.float32))
        else:
            out[k] = draw_normal_bf16(rng, shp, std, bits=bits)
    return out


def draw_weights(cfg_id: int, d: ModelDims, *, random_gains: bool, bits: bool = False,
                 std: float = 0.02) -> dict:
    """Whole model: {'emb','gf','lm','layers':[...]}; untied LM head."""
    rng = workload_seed(cfg_id, "weights", 0)
    w = {
        "emb": draw_normal_bf16(rng, (d.vocab, d.d_model), std, bits=bits),
        "gf": (draw_normal_bf16(rng, (d.d_model,), std, 1.0) if random_gains
               else np.ones((d.d_model,), dtype=np.float32)),
        "lm": draw_normal_bf16(rng, (d.vocab, d.d_model), std, bits=bits),
        "layers": [draw_layer_weights(cfg_id, d, l, random_gains=random_gains, bits=bits, std=std)
                   for l in range(d.n_layers)],
    }
    return w


def draw_prefix_embeddings(cfg_id: int, n_rows: int, d_model: int, extra: int = 0) -> np.ndarray:
    """N(0,1) rows standing in for image-patch / trajectory embeddings."""
    return draw_normal_bf16(workload_seed(cfg_id, "prefix", extra), (n_rows, d_model))


def draw_tokens(cfg_id: int, n: int, vocab: int, extra: int = 0) -> np.ndarray:
    return workload_seed(cfg_id, "tokens", 100 + extra).integers(0, vocab, size=n).astype(np.int32)
