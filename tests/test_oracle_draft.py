"""Pins of the draft-side oracle (CPU only): the tree forward of Cache Construction eq. (1) with
the mask of Mask Construction for Draft Model, and the per-row top-k of eq. (2).

What fixes the expected values: a node's distribution is by definition the model's next-token
distribution after the token sequence from the root of the text to that node, so every tree row
must equal the LAST row of a cache-free recompute of context + root path (a different code path);
a tree that is a chain must equal the causal chain forward; softmax / top-k against torch."""
import numpy as np
import pytest
import torch

import card_inputs as ci
from oracle import card_oracle as co
from oracle.cache_oracle import tree_mask
from oracle.from_inputs import oracle_weights

ODD = ci.ModelShape("odd", 3, 96, 6, 2, 16, 80, 211, rope_theta=100.0, ctx=9, r=5)


def _tree(rng, widths, vocab):
    """levels of (tokens, parents): level 0 has parents -1."""
    levels, prev = [], 0
    for l, n in enumerate(widths):
        toks = rng.integers(0, vocab, size=n).tolist()
        parents = [-1] * n if l == 0 else rng.integers(0, prev, size=n).tolist()
        levels.append((toks, parents))
        prev = n
    return levels


def _paths(levels):
    """token path from level 0 to every node, level by level."""
    out, prev = [], []
    for l, (toks, parents) in enumerate(levels):
        cur = [([] if l == 0 else prev[p]) + [t] for t, p in zip(toks, parents)]
        out.append(cur)
        prev = cur
    return out


@pytest.mark.parametrize("store", ["bf16", "exact"])
def test_tree_rows_equal_cache_free_recompute_of_each_root_path(store):
    cfg = ODD
    rng = np.random.default_rng(4)
    w = oracle_weights(cfg, 4, gain_jitter=0.3)
    ctx = ci.uniform_tokens(4, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    levels = _tree(rng, [3, 5, 4, 6], cfg.vocab)
    mask = tree_mask([p for _, p in levels])
    offs = np.cumsum([0] + [len(t) for t, _ in levels])
    kv = co.OracleKV.empty(cfg, 64, store=store)
    co.prefill(cfg, w, kv, ctx, chunk=4)
    base = 16  # tree slots start at a page boundary behind the context, as on the device
    paths = _paths(levels)
    for l, (toks, parents) in enumerate(levels):
        n = len(toks)
        slots = [base + int(offs[l]) + i for i in range(n)]
        visible = [list(range(cfg.ctx)) + [base + j for j in np.flatnonzero(mask[offs[l] + i])] for i in range(n)]
        logits = co.forward_tree_rows(cfg, w, kv, toks, [cfg.ctx + l] * n, slots, visible)
        for i in range(n):
            ref = co.full_recompute(cfg, w, ctx + paths[l][i], store=store)[-1]
            np.testing.assert_allclose(logits[i], ref, rtol=1e-9, atol=1e-11)
    # peers are invisible: swapping the token of a node changes no row but its own and its descendants'
    assert mask[offs[1] + 1, offs[1] + 2] == False  # noqa: E712


def test_chain_shaped_tree_is_the_causal_chain_forward():
    cfg = ODD
    w = oracle_weights(cfg, 6)
    ctx = ci.uniform_tokens(6, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    cand = ci.uniform_tokens(6, "cand_tokens", 0, 4, cfg.vocab).tolist()
    kv_a = co.OracleKV.empty(cfg, 32)
    co.prefill(cfg, w, kv_a, ctx)
    chain = co.forward_rows(cfg, w, kv_a, cand, cfg.ctx)
    kv_b = co.OracleKV.empty(cfg, 32)
    co.prefill(cfg, w, kv_b, ctx)
    # all four rows in ONE tree call: row i sees the context and rows 0..i
    slots = [cfg.ctx + i for i in range(4)]
    vis = [list(range(cfg.ctx + i + 1)) for i in range(4)]
    tree = co.forward_tree_rows(cfg, w, kv_b, cand, slots, slots, vis)
    np.testing.assert_allclose(tree, chain, rtol=1e-10, atol=1e-12)


def test_softmax_and_topk_against_torch():
    rng = np.random.default_rng(0)
    logits = rng.normal(size=(5, 97)) * 3
    logits[2, 10] = logits[2, 50]  # an exact tie: ascending token order
    p = co.softmax_rows(logits)
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(logits), -1).numpy(), rtol=1e-12)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-12)
    toks, vals = co.topk_rows(p, 7)
    tv, ti = torch.topk(torch.from_numpy(p), 7, dim=-1)
    np.testing.assert_allclose(vals, tv.numpy(), rtol=1e-12)
    for i in range(5):
        assert sorted(toks[i].tolist()) == sorted(ti[i].tolist())
        assert all(vals[i, j] >= vals[i, j + 1] for j in range(6))
    if 10 in toks[2].tolist() and 50 in toks[2].tolist():
        assert toks[2].tolist().index(10) < toks[2].tolist().index(50)
