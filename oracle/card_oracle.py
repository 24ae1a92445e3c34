"""CPU oracle for the target model's chain-verification step of CARD.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file;
it exists so that tests, the smoke check and the benchmark's cpu_baseline leg
can say what the HIP path must compute.  It shares no code with the HIP path.

What it is: the plain definition.  At temperature 0 the method is lossless
(CARD Design, closing sentence of the overview; Fig. 2 caption): the target
runs one chain-shaped (plain causal) forward over the selected candidate path
(Contributions, "Computation Offloading"; Cache Correction, last paragraph),
compares its own arg-max prediction with each candidate, keeps the longest
matching prefix and emits its own next token.  So the oracle is a standard
pre-norm decoder forward (RMSNorm, rotary embedding with half-split pairing,
grouped-query attention, SwiGLU; the model families of Experimental Setup)
followed by that comparison, written row by row with no blocking or fusion.

Floating point: every operation runs in `dtype` (float64 by default; float32
for the full-size shapes, where 64-bit weights do not fit in host memory).
Weights are bf16-representable values widened to `dtype`.  The target's KV
cache is a bf16 cache: what the step stores for later steps (and for its own
later rows) is K after rotation and V rounded to bf16, round-to-nearest-even
from the float32 value; every later use reads that stored value widened to
`dtype`.  That rounding is part of what the step computes, not an error of an
implementation, so the oracle applies it too (`OracleKV.empty(..., store="bf16")`,
the default); `store="exact"` keeps the unrounded values (the textbook decoder,
used by pins that compare with closed forms).

Pins (tests/test_oracle_*.py): row-batched verify == token-by-token decode ==
cache-free full recompute (a separate code path below); planted-prefix
invariant; rotary, norm, softmax and GQA identities; blocks against torch's
CPU library routines; sampling: draw frequencies against the softmax (chi-square),
acceptance rate against p(c), chained steps against token-by-token sampling.
The paper prints no numeric example of a forward pass; the logit values are pinned
by the whole forward rebuilt from torch's CPU library routines and by the cache-free
recompute, the decisions by brute force and the planted prefixes.  No function
of this file is without a pin.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class OracleWeights:
    """Matrices are [out_features, in_features]; `layer(l)` returns the dict
    {wq, wk, wv, wo, wg, wu, wd, g_attn, g_ffn} of layer l (it may build it lazily)."""

    embed: np.ndarray
    lm_head: np.ndarray
    g_final: np.ndarray
    layer: Callable[[int], Dict[str, np.ndarray]]


def round_bf16(x: np.ndarray) -> np.ndarray:
    """x rounded to bfloat16 (8 significant bits), ties to even, via its float32 value;
    returned in x's dtype.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(x.dtype).reshape(x.shape)


def cache_value(x: np.ndarray, store: str) -> np.ndarray:
    """The value a cache of precision `store` ("bf16" or "exact") holds for x."""
    if store == "bf16":
        return round_bf16(x)
    if store == "exact":
        return x
    raise ValueError(store)


@dataclass
class OracleKV:
    """Per layer: K (after rotation) and V for positions [0, capacity), [pos, kv_head, head_dim],
    as the cache holds them (`store`: "bf16" rounds on write, "exact" does not)."""

    k: List[np.ndarray] = field(default_factory=list)
    v: List[np.ndarray] = field(default_factory=list)
    store: str = "bf16"

    @staticmethod
    def empty(cfg, capacity: int, dtype=np.float64, store: str = "bf16") -> "OracleKV":
        shp = (capacity, cfg.n_kv_heads, cfg.head_dim)
        return OracleKV(
            [np.zeros(shp, dtype) for _ in range(cfg.n_layers)],
            [np.zeros(shp, dtype) for _ in range(cfg.n_layers)],
            store,
        )


# --------------------------------------------------------------------------- blocks


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(z: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotary embedding of z[..., h] at integer position pos.  Pair (j, j+h/2) is turned
    by the angle pos * theta^(-2j/h) (half-split pairing, the convention of the
    HuggingFace LLaMA implementation the paper runs on)."""
    h = z.shape[-1]
    half = h // 2
    j = np.arange(half, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * j / h)
    c = np.cos(ang).astype(z.dtype)
    s = np.sin(ang).astype(z.dtype)
    a, b = z[..., :half], z[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def attend_row(cfg, q: np.ndarray, k_hist: np.ndarray, v_hist: np.ndarray) -> np.ndarray:
    """One query position.  q [n_q_heads, h]; k_hist, v_hist [p+1, n_kv_heads, h] hold every
    position the row may see (its own included).  Query head a reads KV head a // G."""
    group = cfg.n_q_heads // cfg.n_kv_heads
    out = np.empty_like(q)
    inv = 1.0 / np.sqrt(np.array(cfg.head_dim, dtype=q.dtype))
    for a in range(cfg.n_q_heads):
        b = a // group
        s = (k_hist[:, b, :] @ q[a]) * inv
        p = softmax(s)
        out[a] = p @ v_hist[:, b, :]
    return out


# --------------------------------------------------------------------------- forward with KV cache


def forward_rows(
    cfg, w: OracleWeights, kv: OracleKV, tokens: Sequence[int], start_pos: int, dtype=np.float64
) -> np.ndarray:
    """Forward len(tokens) rows at positions start_pos.. against kv[0:start_pos); row i also
    sees rows 0..i (plain causal chain).  Writes K and V of every row into kv.  Returns the
    final logits [rows, vocab]."""
    r = len(tokens)
    x = np.stack([w.embed[int(t)].astype(dtype) for t in tokens])
    hq, hkv, h = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    for l in range(cfg.n_layers):
        wl = w.layer(l)
        u = rmsnorm(x, wl["g_attn"].astype(dtype), dtype(cfg.rms_eps))
        q = u @ wl["wq"].astype(dtype).T
        k = u @ wl["wk"].astype(dtype).T
        v = u @ wl["wv"].astype(dtype).T
        att = np.empty((r, hq * h), dtype)
        for i in range(r):
            p = start_pos + i
            qi = rope(q[i].reshape(hq, h), p, cfg.rope_theta)
            kv.k[l][p] = cache_value(rope(k[i].reshape(hkv, h), p, cfg.rope_theta), kv.store)
            kv.v[l][p] = cache_value(v[i].reshape(hkv, h), kv.store)
            att[i] = attend_row(cfg, qi, kv.k[l][: p + 1], kv.v[l][: p + 1]).reshape(-1)
        x = x + att @ wl["wo"].astype(dtype).T
        u2 = rmsnorm(x, wl["g_ffn"].astype(dtype), dtype(cfg.rms_eps))
        gate = u2 @ wl["wg"].astype(dtype).T
        up = u2 @ wl["wu"].astype(dtype).T
        x = x + (silu(gate) * up) @ wl["wd"].astype(dtype).T
    y = rmsnorm(x, w.g_final.astype(dtype), dtype(cfg.rms_eps))
    return y @ w.lm_head.astype(dtype).T


def forward_tree_rows(
    cfg, w: OracleWeights, kv: OracleKV, tokens: Sequence[int], positions: Sequence[int], slots: Sequence[int],
    visible: Sequence[Sequence[int]], dtype=np.float64,
) -> np.ndarray:
    """Draft-side forward over tree nodes (Cache Construction, eq. (1): the draft decodes the K
    sequences of the primary cache in one pass; Mask Construction for Draft Model).  Row i carries
    token tokens[i] at sequence position positions[i] (context length + depth of the node); its key
    and value go to cache slot slots[i]; it attends to the cache slots visible[i] - the committed
    context, the node's ancestors and the node itself, never its peers - which must include
    slots[i].  Rows of one call do not see each other unless listed.  Returns logits [rows, vocab]."""
    r = len(tokens)
    x = np.stack([w.embed[int(t)].astype(dtype) for t in tokens])
    hq, hkv, h = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    for l in range(cfg.n_layers):
        wl = w.layer(l)
        u = rmsnorm(x, wl["g_attn"].astype(dtype), dtype(cfg.rms_eps))
        q = u @ wl["wq"].astype(dtype).T
        k = u @ wl["wk"].astype(dtype).T
        v = u @ wl["wv"].astype(dtype).T
        for i in range(r):  # every row's key and value are stored before any row attends
            kv.k[l][slots[i]] = cache_value(rope(k[i].reshape(hkv, h), positions[i], cfg.rope_theta), kv.store)
            kv.v[l][slots[i]] = cache_value(v[i].reshape(hkv, h), kv.store)
        att = np.empty((r, hq * h), dtype)
        for i in range(r):
            assert slots[i] in visible[i]
            vis = np.asarray(sorted(visible[i]), dtype=np.int64)
            qi = rope(q[i].reshape(hq, h), positions[i], cfg.rope_theta)
            att[i] = attend_row(cfg, qi, kv.k[l][vis], kv.v[l][vis]).reshape(-1)
        x = x + att @ wl["wo"].astype(dtype).T
        u2 = rmsnorm(x, wl["g_ffn"].astype(dtype), dtype(cfg.rms_eps))
        gate = u2 @ wl["wg"].astype(dtype).T
        up = u2 @ wl["wu"].astype(dtype).T
        x = x + (silu(gate) * up) @ wl["wd"].astype(dtype).T
    y = rmsnorm(x, w.g_final.astype(dtype), dtype(cfg.rms_eps))
    return y @ w.lm_head.astype(dtype).T


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """Row-wise softmax: the distributions P_i of eq. (1)."""
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def topk_rows(probs: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (2): per row the k most probable tokens and their probabilities, most probable first;
    equal probabilities in ascending token order."""
    toks = np.empty((probs.shape[0], k), dtype=np.int64)
    vals = np.empty((probs.shape[0], k), dtype=probs.dtype)
    for i, row in enumerate(probs):
        order = sorted(range(row.shape[0]), key=lambda t: (-row[t], t))[:k]
        toks[i] = order
        vals[i] = row[order]
    return toks, vals


def prefill(cfg, w, kv, ctx_tokens: Sequence[int], dtype=np.float64, chunk: int = 64) -> int:
    """Fill kv[0:n) from the context and return the pending prediction g0 = arg-max of the
    last context row."""
    n = len(ctx_tokens)
    last = None
    for s in range(0, n, chunk):
        last = forward_rows(cfg, w, kv, ctx_tokens[s : s + chunk], s, dtype)
    return int(argmax_lowest(last[-1]))


def argmax_lowest(row: np.ndarray) -> int:
    """Index of the maximum; the lowest index on exact ties."""
    return int(np.argmax(row))


def top2_gap(row: np.ndarray) -> float:
    """Largest minus second-largest logit of one row."""
    part = np.partition(row, -2)
    return float(part[-1] - part[-2])


# --------------------------------------------------------------------------- sampling


def _mix32(x: np.ndarray) -> np.ndarray:
    """32-bit xorshift-multiply finaliser ("lowbias32", C. Wellons, public domain) on uint64 lanes."""
    m = np.uint64(0xFFFFFFFF)
    x = x & m
    x = x ^ (x >> np.uint64(16))
    x = (x * np.uint64(0x7FEB352D)) & m
    x = x ^ (x >> np.uint64(15))
    x = (x * np.uint64(0x846CA68B)) & m
    x = x ^ (x >> np.uint64(16))
    return x


def gumbel_noise(seed: int, pos: int, vocab: int) -> np.ndarray:
    """Standard Gumbel noise G[v], v in [0, vocab), for the token drawn at absolute position pos:
    a counter-based generator (the draw for a position must not depend on which step computes
    it).  key = mix(mix(mix(seed_lo ^ 0x243f6a88) ^ seed_hi) ^ pos); h = mix(key + v * 0x9e3779b9);
    u = ((h >> 8) + 1/2) / 2^24 in (0, 1); G = -ln(-ln u)."""
    lo, hi = np.uint64(seed & 0xFFFFFFFF), np.uint64((seed >> 32) & 0xFFFFFFFF)
    key = _mix32(_mix32(_mix32(np.array([lo ^ np.uint64(0x243F6A88)], dtype=np.uint64)) ^ hi) ^ np.uint64(pos & 0xFFFFFFFF))
    v = np.arange(vocab, dtype=np.uint64)
    h = _mix32((key + v * np.uint64(0x9E3779B9)) & np.uint64(0xFFFFFFFF))
    u = ((h >> np.uint64(8)).astype(np.float64) + 0.5) / 16777216.0
    return -np.log(-np.log(u))


def perturbed(row: np.ndarray, pos: int, temperature: float, seed: int) -> np.ndarray:
    """logits / T + G(seed, pos, .): its arg-max is a draw from softmax(logits / T) (the maximum of
    independently Gumbel-shifted scores falls on index v with probability softmax(score)[v]).
    Temperature 0 returns the logits themselves (greedy)."""
    if temperature <= 0.0:
        return row
    return row.astype(np.float64) / temperature + gumbel_noise(seed, pos, row.shape[0])


# --------------------------------------------------------------------------- acceptance


@dataclass
class VerifyResult:
    accepted_len: int
    correction_token: int
    kv_first_slot: int
    kv_count: int
    row_argmax: List[int]
    row_gap: List[float]
    logits: Optional[np.ndarray] = None


def greedy_accept(pending: int, row_argmax: Sequence[int], cand: Sequence[int]) -> Tuple[int, int]:
    """Greedy (temperature 0) acceptance over a chain of r candidates.

    pred[0] is the pending prediction for the first candidate's position (a negative value
    means "none: take the first candidate as given"); pred[i] is the arg-max of row i-1.  The
    accepted length is the longest prefix on which candidate and prediction agree; the
    correction token is the target's own prediction right after it (Fig. 2: after the accepted
    path the target emits its next token; after a rejection it emits the replacement)."""
    r = len(cand)
    pred = [int(cand[0]) if pending < 0 else int(pending)] + [int(a) for a in row_argmax]
    j = 0
    while j < r and int(cand[j]) == pred[j]:
        j += 1
    return j, pred[j]


def verify(
    cfg, w, kv, ctx_len: int, pending: int, cand: Sequence[int], dtype=np.float64, keep_logits=False,
    temperature: float = 0.0, seed: int = 0,
) -> VerifyResult:
    """One verification step: forward the r candidates at positions ctx_len.., then accept.

    Temperature 0 (the paper's main setting): the target's token after row i is the arg-max of
    row i.  Temperature > 0 (the T = 1 columns of the main results; the paper states only that the
    sampling mechanism of speculative decoding is kept): the cached path is a deterministic
    proposal, for which speculative sampling accepts candidate c with probability p(c) and
    otherwise emits a draw from p restricted to the other tokens; one draw x ~ p per position
    gives both (accept iff x == c, else emit x).  Row i's draw is for position ctx_len + i + 1 and
    uses that position's noise, so the same prefix rule applies with draws in place of arg-maxes.
    row_argmax / row_gap then hold the draws and the top-1/top-2 gaps of the perturbed rows."""
    logits = forward_rows(cfg, w, kv, cand, ctx_len, dtype)
    scored = [perturbed(row, ctx_len + i + 1, temperature, seed) for i, row in enumerate(logits)]
    am = [argmax_lowest(row) for row in scored]
    gaps = [top2_gap(row) for row in scored]
    j, corr = greedy_accept(pending, am, cand)
    return VerifyResult(j, corr, ctx_len, j, am, gaps, logits if keep_logits else None)


# --------------------------------------------------------------------------- cache-free recompute


def full_recompute(cfg, w: OracleWeights, tokens: Sequence[int], dtype=np.float64, store: str = "bf16") -> np.ndarray:
    """Logits [T, vocab] of the whole sequence from scratch: no KV cache, one dense causal mask,
    attention as a masked T x T matrix per head.  Deliberately a different code path from
    forward_rows (whole-sequence tensors, explicit mask, explicit repetition of KV heads).
    K and V enter attention as a cache of precision `store` would hold them."""
    t_len = len(tokens)
    hq, hkv, h = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    group = hq // hkv
    x = w.embed[np.asarray(tokens, dtype=np.int64)].astype(dtype)
    pos = np.arange(t_len, dtype=np.float64)
    inv_freq = cfg.rope_theta ** (-np.arange(0, h, 2, dtype=np.float64) / h)
    ang = pos[:, None] * inv_freq[None, :]
    cos = np.cos(ang).astype(dtype)[:, None, :]
    sin = np.sin(ang).astype(dtype)[:, None, :]

    def rot(z):  # z [T, heads, h]
        z1, z2 = z[..., : h // 2], z[..., h // 2 :]
        return np.concatenate([z1 * cos - z2 * sin, z2 * cos + z1 * sin], axis=-1)

    mask = np.where(np.tril(np.ones((t_len, t_len), dtype=bool)), 0.0, -np.inf).astype(dtype)
    for l in range(cfg.n_layers):
        wl = w.layer(l)
        u = rmsnorm(x, wl["g_attn"].astype(dtype), dtype(cfg.rms_eps))
        q = rot((u @ wl["wq"].astype(dtype).T).reshape(t_len, hq, h))
        k = cache_value(rot((u @ wl["wk"].astype(dtype).T).reshape(t_len, hkv, h)), store)
        v = cache_value((u @ wl["wv"].astype(dtype).T).reshape(t_len, hkv, h), store)
        k = np.repeat(k, group, axis=1)
        v = np.repeat(v, group, axis=1)
        s = np.einsum("iah,jah->aij", q, k) / np.sqrt(dtype(h)) + mask[None]
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        att = np.einsum("aij,jah->iah", p, v).reshape(t_len, hq * h)
        x = x + att @ wl["wo"].astype(dtype).T
        u2 = rmsnorm(x, wl["g_ffn"].astype(dtype), dtype(cfg.rms_eps))
        x = x + (silu(u2 @ wl["wg"].astype(dtype).T) * (u2 @ wl["wu"].astype(dtype).T)) @ wl[
            "wd"
        ].astype(dtype).T
    y = rmsnorm(x, w.g_final.astype(dtype), dtype(cfg.rms_eps))
    return y @ w.lm_head.astype(dtype).T


def greedy_decode_bruteforce(
    cfg, w, ctx_tokens: Sequence[int], n_new: int, dtype=np.float64, store: str = "bf16",
    temperature: float = 0.0, seed: int = 0,
) -> List[int]:
    """Plain autoregressive decoding, one token at a time, recomputing the whole sequence each
    time: greedy at temperature 0, else sampling (the token at position p is the arg-max of the
    last row's logits / T + G(seed, p, .)).  Returns [g0, g1, ..., g_{n_new-1}]."""
    seq = [int(t) for t in ctx_tokens]
    out = []
    for _ in range(n_new):
        logits = full_recompute(cfg, w, seq, dtype, store)
        nxt = argmax_lowest(perturbed(logits[-1], len(seq), temperature, seed))
        out.append(nxt)
        seq.append(nxt)
    return out


def greedy_decode_cached(cfg, w, kv, ctx_len: int, pending: int, n_new: int, dtype=np.float64,
                         temperature: float = 0.0, seed: int = 0):
    """Autoregressive decoding with the KV cache (greedy, or sampling at a temperature > 0): feeds
    the pending token, then each prediction in turn.  Returns ([pending, g1, ..., g_{n_new}], gaps
    of g1..; at a temperature the gaps of the perturbed rows)."""
    toks = [int(pending)]
    gaps = []
    for i in range(n_new):
        logits = forward_rows(cfg, w, kv, [toks[-1]], ctx_len + i, dtype)
        row = perturbed(logits[0], ctx_len + i + 1, temperature, seed)
        toks.append(argmax_lowest(row))
        gaps.append(top2_gap(row))
    return toks, gaps
