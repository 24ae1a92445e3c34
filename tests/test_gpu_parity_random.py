"""Randomly drawn small configurations against the oracle: model widths (head size 64 / 128, one
to four KV heads, one to seven query heads per KV head, FFN and vocabulary sizes that are no
multiple of a tile), depth, context length (empty, around page and cut boundaries, up to 6000
tokens), r on both sides of every tile boundary, the caller's grid size, the prefill piece
size and the page placement are all drawn from a seeded generator; the bars are those of the
other parity tests (logits 2e-2 of the row maximum, decisions bit-exact where decisive, keys and
values within a bf16 step).  The same for the draft-side tree forward with random trees."""
import numpy as np
import pytest

import card_inputs as ci
from gpu_common import GAP, logits_rel_err, shuffled_pages
from oracle import card_oracle as co
from oracle.cache_oracle import tree_mask
from oracle.from_inputs import oracle_weights

pytestmark = pytest.mark.gpu


def _model(rng, tag):
    h = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 4, 7]))
    return dict(name=tag, n_layers=int(rng.integers(1, 4)), d_model=64 * int(rng.integers(2, 11)), n_q_heads=hkv * g,
                n_kv_heads=hkv, head_dim=h, d_ffn=8 * int(rng.integers(8, 260)), vocab=int(rng.integers(40, 5000)))


def _pair(shape, seed, max_ctx, grid):
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    tgt = card.Target(shape, max_ctx, max_r=32, grid_wgs=grid, page_order=shuffled_pages(max_ctx // 16, seed))
    load_synthetic_weights(tgt, shape, seed, 0.2)
    return tgt, oracle_weights(shape, seed, 0.2)


@pytest.mark.parametrize("batch", range(4))
def test_verify_step_on_random_configurations(batch):
    rng = np.random.default_rng(1000 + batch)
    for case in range(10):
        m = _model(rng, f"random-{batch}-{case}")
        r = int(rng.choice([1, 2, 3, 5, 8, 9, 12, 16, 17, 24, 31, 32]))
        ctx_len = int(rng.choice([0, 1, 15, 16, 17, int(rng.integers(0, 300)), int(rng.integers(300, 700)), 511, 512, 513,
                                  int(rng.integers(700, 1400)), int(rng.integers(1400, 6000)), 4095, 4096, 4097]))
        grid = int(rng.choice([0, 256, 192, 128, 100, 64, 40, 24, 8, 252]))
        chunk = int(rng.choice([7, 16, 29, 32]))
        seed = int(rng.integers(1, 1000))
        shape = ci.ModelShape(ctx=ctx_len, r=r, **m)
        max_ctx = (ctx_len + r + 15) // 16 * 16 + 16 * int(rng.integers(0, 3))
        what = f"{m} ctx {ctx_len} r {r} grid {grid} chunk {chunk} seed {seed}"
        print(what, flush=True)
        tgt, w = _pair(shape, seed, max_ctx, grid)
        toks = ci.uniform_tokens(seed, "ctx_tokens", r, ctx_len + r, shape.vocab).tolist()
        kv = co.OracleKV.empty(shape, max_ctx)
        if ctx_len:
            co.prefill(shape, w, kv, toks[:ctx_len], chunk=256)
            tgt.prefill(toks[:ctx_len], chunk=chunk)
        ref = co.verify(shape, w, kv, ctx_len, -1, toks[ctx_len:], keep_logits=True)
        res = tgt.verify(ctx_len, -1, toks[ctx_len:], want_logits=True)
        assert logits_rel_err(res["logits"], ref.logits) <= 2e-2, what
        for i, row in enumerate(ref.logits):
            top2 = np.argsort(row)[-2:][::-1]
            if co.top2_gap(row) > GAP:
                assert res["row_argmax"][i] == int(top2[0]), (what, i)
            else:
                assert res["row_argmax"][i] in (int(top2[0]), int(top2[1])), (what, i)
        if all(gap > GAP for gap in ref.row_gap[: ref.accepted_len]):
            assert (res["accepted_len"], res["correction_token"]) == (ref.accepted_len, ref.correction_token), what
        k, v = tgt.kv_gather(shape.n_layers - 1, 0, ctx_len + r)
        ref_k, ref_v = kv.k[-1][: ctx_len + r], kv.v[-1][: ctx_len + r]
        assert np.abs(k.numpy() - ref_k).max() <= 2.0 ** -7 * np.abs(ref_k).max(), what
        assert np.abs(v.numpy() - ref_v).max() <= 2.0 ** -7 * np.abs(ref_v).max(), what
        del tgt


@pytest.mark.parametrize("batch", range(2))
def test_draft_level_on_random_trees_and_configurations(batch):
    import paper_2508_04462_amd as card
    from test_gpu_draft import _check_topk, _levels

    rng = np.random.default_rng(2000 + batch)
    for case in range(10):
        m = _model(rng, f"random-tree-{batch}-{case}")
        ctx_len = int(rng.choice([0, 1, 16, 37, int(rng.integers(0, 300)), int(rng.integers(300, 1200)), 512]))
        widths = [int(rng.integers(1, 41)) for _ in range(int(rng.integers(1, 5)))]
        k = int(rng.integers(1, min(16, m["vocab"] - 1) + 1))
        grid = int(rng.choice([0, 256, 192, 128, 100, 64, 40, 24, 8]))
        seed = int(rng.integers(1, 1000))
        shape = ci.ModelShape(ctx=ctx_len, r=4, **m)
        mask_base, tree_base = ctx_len // 16 * 16, (ctx_len + 15) // 16 * 16
        max_ctx = (tree_base + sum(widths) + 15) // 16 * 16 + 16
        what = f"{m} ctx {ctx_len} widths {widths} k {k} grid {grid} seed {seed}"
        print(what, flush=True)
        tgt, w = _pair(shape, seed, max_ctx, grid)
        ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
        kv = co.OracleKV.empty(shape, max_ctx)
        if ctx_len:
            co.prefill(shape, w, kv, ctx, chunk=256)
            tgt.prefill(ctx, chunk=29)
        levels = _levels(np.random.default_rng(seed), widths, shape.vocab)
        ref_mask = tree_mask([p for _, p in levels])
        offs = np.cumsum([0] + widths)
        words = (tree_base + int(offs[-1]) - mask_base + 31) // 32
        prev_rows = None
        for l, (toks, parents) in enumerate(levels):
            n, first = len(toks), tree_base + int(offs[l])
            st, rows = card.card_tree_mask_level(prev_rows, parents, first, ctx_len, mask_base, words)
            assert st == card.CARD_OK, what
            visible = [list(range(ctx_len)) + [tree_base + int(j) for j in np.flatnonzero(ref_mask[offs[l] + i])]
                       for i in range(n)]
            ref = co.forward_tree_rows(shape, w, kv, toks, [ctx_len + l] * n, [first + i for i in range(n)], visible)
            for c0 in range(0, n, 32):
                c1 = min(n, c0 + 32)
                res = tgt.draft_level(ctx_len, toks[c0:c1], [ctx_len + l] * (c1 - c0), first + c0, rows[c0:c1], mask_base,
                                      k, want_logits=True)
                assert logits_rel_err(res["logits"], ref[c0:c1]) <= 2e-2, what
                tk, tp = res["topk_tokens"].cpu().numpy(), res["topk_probs"].cpu().double().numpy()
                for i in range(c0, c1):
                    _check_topk(tk[i - c0], tp[i - c0], ref[i], k)
            prev_rows = rows
            kk, _ = tgt.kv_gather(shape.n_layers - 1, first, n)
            assert np.abs(kk.numpy() - kv.k[-1][first: first + n]).max() <= 2.0 ** -7 * np.abs(kv.k[-1][: first + n]).max(), what
        del tgt
