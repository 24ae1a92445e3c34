"""Counter-based generators: integer hashing only, identical on CPU and GPU.

Matrix entries approximate N(0, std^2): the sum of eight independent 16-bit
uniforms (Irwin-Hall, n = 8; |z| <= 4.9 sigma, excess kurtosis -0.15), centred,
scaled in fp32 and rounded once to bf16.  No libm call is involved, so a torch
CPU tensor and a torch GPU tensor made from the same (seed, tag, layer) hold
the same bits.  The 32-bit mixer is the two-multiply xorshift finaliser
"lowbias32" published by C. Wellons (hash-prospector, public domain).
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import torch

from .configs import ModelShape

_M32 = 0xFFFFFFFF
_GOLD = 0x9E3779B9

# tag -> small integer mixed into the stream key; fixed forever (goldens depend on it)
TENSOR_TAGS: Dict[str, int] = {
    "embed": 1,
    "wq": 2,
    "wk": 3,
    "wv": 4,
    "wo": 5,
    "wg": 6,
    "wu": 7,
    "wd": 8,
    "lm_head": 9,
    "g_attn": 10,
    "g_ffn": 11,
    "g_final": 12,
    "ctx_tokens": 13,
    "cand_tokens": 14,
    "kv_noise": 15,
    "misc": 16,
}


def _mix32_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & _M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & _M32
    x ^= x >> 16
    return x


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """x: int64 tensor with values in [0, 2^32).  Returns the same."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    # the second constant exceeds 2^31: split the operand so no product reaches 2^63
    lo = (x & 0xFFFF) * 0x846CA68B
    hi = (((x >> 16) * 0x846CA68B) & 0xFFFF) << 16
    x = (lo + hi) & _M32
    x = x ^ (x >> 16)
    return x


def stream_key(seed: int, tag: str, layer: int = 0) -> int:
    """32-bit key of one tensor's random stream."""
    k = _mix32_int(seed ^ 0x5BD1E995)
    k = _mix32_int(k ^ (TENSOR_TAGS[tag] * _GOLD))
    k = _mix32_int(k ^ ((layer + 1) * 0x85EBCA6B))
    return k


def _hash_words(idx: torch.Tensor, key: int, n_words: int) -> List[torch.Tensor]:
    a = _mix32(idx ^ key)
    return [_mix32((a + (j + 1) * _GOLD) & _M32) for j in range(n_words)]


_IH8_STD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)


def _irwin_hall8(idx: torch.Tensor, key: int) -> torch.Tensor:
    """Centred integer sum of eight 16-bit uniforms, as fp32 (exact: |s| < 2^19)."""
    s = torch.zeros_like(idx)
    for w in _hash_words(idx, key, 4):
        s = s + (w & 0xFFFF) + (w >> 16)
    return (s - 4 * 65535).to(torch.float32)


def bf16_matrix(
    seed: int,
    tag: str,
    layer: int,
    rows: int,
    cols: int,
    std: float = 0.02,
    device: str | torch.device = "cpu",
    chunk_rows: int | None = None,
) -> torch.Tensor:
    """[rows, cols] bf16, entry (i, j) drawn from stream (seed, tag, layer) at counter i*cols+j."""
    assert rows * cols < 2 ** 32
    key = stream_key(seed, tag, layer)
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 24) // cols)
    scale = std / _IH8_STD
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        idx = torch.arange(r0 * cols, r1 * cols, dtype=torch.int64, device=device)
        z = _irwin_hall8(idx, key) * scale
        out[r0:r1] = z.to(torch.bfloat16).view(r1 - r0, cols)
    return out


def gains(
    seed: int,
    tag: str,
    layer: int,
    n: int,
    jitter: float = 0.0,
    device: str | torch.device = "cpu",
) -> torch.Tensor:
    """RMSNorm gains, fp32 [n].  jitter = 0 gives exactly 1.0 (the workload recipe);
    tests use jitter > 0 (gain = 1 + jitter * u, u uniform in [-1, 1) on a 2^-16 grid)
    so that a misplaced or dropped gain is visible."""
    if jitter == 0.0:
        return torch.ones(n, dtype=torch.float32, device=device)
    key = stream_key(seed, tag, layer)
    idx = torch.arange(n, dtype=torch.int64, device=device)
    w = _hash_words(idx, key, 1)[0]
    u = ((w >> 16) - 32768).to(torch.float32) * (1.0 / 32768.0)
    return 1.0 + jitter * u


def uniform_tokens(
    seed: int, tag: str, stream: int, n: int, vocab: int, device: str | torch.device = "cpu"
) -> torch.Tensor:
    """n token ids uniform in [0, vocab), int32."""
    key = stream_key(seed, tag, stream)
    idx = torch.arange(n, dtype=torch.int64, device=device)
    w = _hash_words(idx, key, 1)[0]
    return ((w * vocab) >> 32).to(torch.int32)


def layer_matrices(
    shape: ModelShape, seed: int, layer: int, device: str | torch.device = "cpu", std: float = 0.02
) -> Dict[str, torch.Tensor]:
    """The seven projection matrices of one decoder layer, each [out_features, in_features] bf16."""
    d, f = shape.d_model, shape.d_ffn
    dims = {
        "wq": (shape.q_dim, d),
        "wk": (shape.kv_dim, d),
        "wv": (shape.kv_dim, d),
        "wo": (d, shape.q_dim),
        "wg": (f, d),
        "wu": (f, d),
        "wd": (d, f),
    }
    return {t: bf16_matrix(seed, t, layer, rc[0], rc[1], std, device) for t, rc in dims.items()}


def plant_candidates(
    greedy: Sequence[int], j: int, r: int, vocab: int, seed: int, stream: int = 0
) -> List[int]:
    """Candidate tokens with a planted matching prefix of length exactly j.

    greedy[i] is the token the target itself would emit at position ctx_len+i
    (greedy[0] is the pending prediction).  c[0..j) copy it; c[j] is a uniform
    draw forced to differ from greedy[j]; the rest are uniform draws.
    """
    assert 0 <= j <= r and len(greedy) >= min(j + 1, r)
    draws = uniform_tokens(seed, "cand_tokens", stream, r, vocab).tolist()
    cand = [int(t) for t in draws]
    for i in range(j):
        cand[i] = int(greedy[i])
    if j < r and cand[j] == int(greedy[j]):
        cand[j] = (cand[j] + 1) % vocab
    return cand
