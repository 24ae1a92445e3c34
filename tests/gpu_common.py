"""Shared set-up of the GPU parity tests: a Target (HIP path) and the oracle on the same seed."""
from __future__ import annotations

import numpy as np
import torch

import card_inputs as ci
from oracle import card_oracle as co
from oracle.from_inputs import oracle_weights

GAP = 0.05  # decisions are compared bit-exactly only where top-1 beats top-2 by more than this


def shuffled_pages(n_pages: int, seed: int):
    order = np.random.default_rng(seed).permutation(n_pages)
    return [int(p) for p in order]


def make_pair(shape, seed, max_ctx, gain_jitter=0.0, dtype=np.float64, shuffle=True, max_r=32, pool_fill=None):
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    n_pages = (max_ctx + 15) // 16
    tgt = card.Target(shape, max_ctx, max_r=max_r, page_order=shuffled_pages(n_pages, seed) if shuffle else None,
                      pool_fill=pool_fill)
    load_synthetic_weights(tgt, shape, seed, gain_jitter)
    w = oracle_weights(shape, seed, gain_jitter, dtype=dtype)
    return tgt, w


def logits_rel_err(gpu_logits: torch.Tensor, ref: np.ndarray) -> float:
    """Per row: max |gpu - ref| / max |ref|; returns the worst row."""
    g = gpu_logits.double().numpy()
    return float(np.max(np.abs(g - ref).max(axis=1) / np.abs(ref).max(axis=1)))
