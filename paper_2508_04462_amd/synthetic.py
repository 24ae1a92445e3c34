"""Fills a Target with the seeded synthetic weights of card_inputs (generated on the device,
layer by layer, so that the 70B-shaped model never exists twice in memory)."""
from __future__ import annotations

import card_inputs as ci

from .runtime import Target


def load_synthetic_weights(target: Target, shape, seed: int, gain_jitter: float = 0.0) -> None:
    dev = target.device
    target.pack("embed", 0, ci.bf16_matrix(seed, "embed", 0, shape.vocab, shape.d_model, device=dev))
    target.pack("lm_head", 0, ci.bf16_matrix(seed, "lm_head", 0, shape.vocab, shape.d_model, device=dev))
    target.pack("g_final", 0, ci.gains(seed, "g_final", 0, shape.d_model, gain_jitter, device=dev))
    for l in range(shape.n_layers):
        for name, mat in ci.layer_matrices(shape, seed, l, device=dev).items():
            target.pack(name, l, mat)
        target.pack("g_attn", l, ci.gains(seed, "g_attn", l, shape.d_model, gain_jitter, device=dev))
        target.pack("g_ffn", l, ci.gains(seed, "g_ffn", l, shape.d_model, gain_jitter, device=dev))
