"""Glue: turn the seeded synthetic tensors of `card_inputs` into OracleWeights.

TEST INFRASTRUCTURE ONLY.  No arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

import card_inputs as ci
from .card_oracle import OracleWeights


def _np(t: torch.Tensor, dtype) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float32).numpy().astype(dtype, copy=False)


def oracle_weights(
    shape: ci.ModelShape,
    seed: int,
    gain_jitter: float = 0.0,
    dtype=np.float64,
    cache_layers: bool = True,
    device: str = "cpu",
) -> OracleWeights:
    """Weights of `shape` from `seed`.  Layers are generated on first use; with
    cache_layers=False they are regenerated on every use (full-size shapes)."""
    store: Dict[int, Dict[str, np.ndarray]] = {}

    def layer(l: int) -> Dict[str, np.ndarray]:
        if l in store:
            return store[l]
        mats = ci.layer_matrices(shape, seed, l, device=device)
        out = {k: _np(v, dtype) for k, v in mats.items()}
        out["g_attn"] = _np(ci.gains(seed, "g_attn", l, shape.d_model, gain_jitter), dtype)
        out["g_ffn"] = _np(ci.gains(seed, "g_ffn", l, shape.d_model, gain_jitter), dtype)
        if cache_layers:
            store[l] = out
        return out

    embed = _np(ci.bf16_matrix(seed, "embed", 0, shape.vocab, shape.d_model, device=device), dtype)
    lm_head = _np(ci.bf16_matrix(seed, "lm_head", 0, shape.vocab, shape.d_model, device=device), dtype)
    g_final = _np(ci.gains(seed, "g_final", 0, shape.d_model, gain_jitter), dtype)
    return OracleWeights(embed, lm_head, g_final, layer)
