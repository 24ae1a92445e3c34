"""Draft-side cache construction on the device against the CPU oracle (Cache Construction,
eqs. (1)-(9); Mask Construction for Draft Model): card_draft_level (tree forward with the
ancestor mask, fused per-row top-k and probabilities) and card_cache_select (path scores and the
global top-K), through the C ABI.

Bars: logits within 2e-2 of the row maximum (as for the verify step); log-probabilities of the
returned tokens within 5e-3 of the oracle's; the returned token SET equals the oracle's top-k
wherever the k-th and (k+1)-th oracle logits are more than 0.05 apart, and the order of two
neighbours is checked wherever they are that far apart; selected tuples equal the oracle's
wherever the scores around the cut and between neighbours are decisive."""
import numpy as np
import pytest
import torch

import card_inputs as ci
from gpu_common import logits_rel_err, make_pair
from oracle import card_oracle as co
from oracle.cache_oracle import build_level, tree_mask

pytestmark = pytest.mark.gpu
TINY = ci.SHAPES["tiny"]
MID = ci.ModelShape("mid", 3, 512, 8, 2, 128, 1048, 3001, ctx=200, r=8)
GAP = 0.05


def _check_topk(tk, tp, ref_logits, k):
    """tk, tp: device results of one row; ref_logits: the oracle's row."""
    order = sorted(range(ref_logits.shape[0]), key=lambda t: (-ref_logits[t], t))
    lse = np.log(np.exp(ref_logits - ref_logits.max()).sum()) + ref_logits.max()
    toks = tk.tolist()
    assert len(set(toks)) == k and all(0 <= t < ref_logits.shape[0] for t in toks)
    for j, t in enumerate(toks):  # probabilities of whatever was returned
        assert abs(np.log(tp[j]) - (ref_logits[t] - lse)) <= 5e-3, (j, t)
    if ref_logits[order[k - 1]] - ref_logits[order[k]] > GAP:
        assert set(toks) == set(order[:k])
    n_ord = 0
    for j in range(k - 1):
        assert tp[j] >= tp[j + 1]
        if ref_logits[order[j]] - ref_logits[order[j + 1]] > GAP and all(
                abs(ref_logits[order[i]] - ref_logits[order[i + 1]]) > GAP for i in range(max(0, j - 1), min(k, j + 2))):
            n_ord += int(toks[j] == order[j])
    return n_ord


def _levels(rng, widths, vocab):
    out, prev = [], 0
    for l, n in enumerate(widths):
        toks = rng.integers(0, vocab, size=n).tolist()
        parents = [-1] * n if l == 0 else rng.integers(0, prev, size=n).tolist()
        out.append((toks, parents))
        prev = n
    return out


@pytest.mark.parametrize("shape,ctx_len,widths,k", [(TINY, 37, [3, 5, 4, 6], 4), (MID, 61, [2, 8, 17, 32], 10),
                                                    (MID, 16, [40], 16), (TINY, 100, [9, 33, 12], 7)],
                         ids=["tiny", "mid", "mid-wide-level", "tiny-wide"])
def test_draft_level_against_the_oracle(shape, ctx_len, widths, k):
    tgt, w = make_pair(shape, 9, max_ctx=320, gain_jitter=0.2)
    rng = np.random.default_rng(9)
    ctx = ci.uniform_tokens(9, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    kv = co.OracleKV.empty(shape, 320)
    co.prefill(shape, w, kv, ctx)
    tgt.prefill(ctx, chunk=29)
    levels = _levels(rng, widths, shape.vocab)
    ref_mask = tree_mask([p for _, p in levels])
    offs = np.cumsum([0] + widths)
    mask_base, tree_base = ctx_len // 16 * 16, (ctx_len + 15) // 16 * 16
    words = (tree_base + int(offs[-1]) - mask_base + 31) // 32
    import paper_2508_04462_amd as card

    prev_rows, n_ord = None, 0
    for l, (toks, parents) in enumerate(levels):
        n = len(toks)
        first = tree_base + int(offs[l])
        st, rows = card.card_tree_mask_level(prev_rows, parents, first, ctx_len, mask_base, words)
        assert st == card.CARD_OK
        visible = [list(range(ctx_len)) + [tree_base + int(j) for j in np.flatnonzero(ref_mask[offs[l] + i])] for i in range(n)]
        ref = co.forward_tree_rows(shape, w, kv, toks, [ctx_len + l] * n, [first + i for i in range(n)], visible)
        for c0 in range(0, n, 32):  # a level wider than 32 rows takes several calls
            c1 = min(n, c0 + 32)
            res = tgt.draft_level(ctx_len, toks[c0:c1], [ctx_len + l] * (c1 - c0), first + c0, rows[c0:c1], mask_base, k,
                                  want_logits=True)
            assert logits_rel_err(res["logits"], ref[c0:c1]) <= 2e-2
            tk, tp = res["topk_tokens"].cpu().numpy(), res["topk_probs"].cpu().double().numpy()
            for i in range(c0, c1):
                n_ord += _check_topk(tk[i - c0], tp[i - c0], ref[i], k)
        prev_rows = rows
        # the keys the level wrote are the oracle's (last layer, first rows)
        kk, vv = tgt.kv_gather(shape.n_layers - 1, first, min(n, 8))
        ref_k = kv.k[-1][first: first + min(n, 8)]
        assert np.abs(kk.numpy() - ref_k).max() <= 2.0 ** -7 * np.abs(ref_k).max()
    assert n_ord > 0


def test_select_exact_on_dyadic_scores_with_ties():
    """eqs. (3)-(7) on inputs whose products are exact in fp32: the result must equal the oracle's
    tuple for tuple, ties included (equal scores in parent, then rank order)."""
    import paper_2508_04462_amd as card

    rng = np.random.default_rng(1)
    for M, k, K in [(5, 4, 7), (50, 10, 50), (100, 16, 100), (3, 2, 10)]:
        vocab = 64
        probs = np.zeros((M, vocab))
        toks = np.zeros((M, k), dtype=np.int32)
        pv = np.zeros((M, k), dtype=np.float32)
        for i in range(M):
            vals = np.sort(rng.integers(1, 16, size=k))[::-1] / 64.0  # few distinct values: many ties
            ids = np.sort(rng.choice(vocab, size=k, replace=False))
            # descending probability, ascending token among equals: what eq. (2) hands over
            order = sorted(range(k), key=lambda j: (-vals[j], ids[j]))
            toks[i], pv[i] = ids[order], vals[order]
            probs[i, ids] = vals
        sigma = (rng.integers(1, 8, size=M) / 8.0).astype(np.float32)
        rt, rs, rp = build_level(probs, sigma.astype(np.float64), K, k)
        dev = "cuda:0"
        ot = torch.empty(K, dtype=torch.int32, device=dev)
        os_ = torch.empty(K, dtype=torch.float32, device=dev)
        op = torch.empty(K, dtype=torch.int32, device=dev)
        n = card.card_cache_select(torch.from_numpy(sigma).to(dev), torch.from_numpy(toks).to(dev),
                                   torch.from_numpy(pv).to(dev), M, k, K, ot, os_, op)
        torch.cuda.synchronize()
        assert n == min(K, M * k) == len(rt)
        assert ot[:n].tolist() == rt.tolist() and op[:n].tolist() == rp.tolist()
        np.testing.assert_array_equal(os_[:n].cpu().numpy().astype(np.float64), rs)
    # parents switched off by a negative token take no part; outputs behind the last tuple are marked empty
    M, k, K, dev = 6, 3, 8, "cuda:0"
    toks = torch.arange(M * k, dtype=torch.int32, device=dev).reshape(M, k)
    toks[[0, 1, 3, 5]] = -1
    pv = torch.tensor([[0.5, 0.25, 0.125]] * M, dtype=torch.float32, device=dev)
    sigma = torch.tensor([1.0, 1.0, 0.5, 1.0, 1.0, 1.0], dtype=torch.float32, device=dev)
    ot = torch.empty(K, dtype=torch.int32, device=dev)
    os_ = torch.empty(K, dtype=torch.float32, device=dev)
    op = torch.empty(K, dtype=torch.int32, device=dev)
    assert card.card_cache_select(sigma, toks, pv, M, k, K, ot, os_, op) == K
    torch.cuda.synchronize()
    # equal scores: the lower parent index first
    assert ot.tolist() == [12, 6, 13, 7, 14, 8, -1, -1] and op.tolist() == [4, 2, 4, 2, 4, 2, -1, -1]
    assert os_.tolist() == [0.5, 0.25, 0.25, 0.125, 0.125, 0.0625, 0.0, 0.0]
    bad = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    assert card.card_cache_select(bad, bad, bad, 200, 16, 10, bad, bad, bad) == card.CARD_ERANGE


def test_three_levels_built_on_the_device_and_written_to_the_cache():
    """Cache construction end to end: level after level, the device expands the current nodes
    (card_draft_level), scores and selects the next level (card_cache_select), the host stores it
    (card_cache_write) and derives the next mask rows; the oracle does the same from its own
    distributions.  Levels are compared while every choice up to them is decisive."""
    import paper_2508_04462_amd as card

    shape, ctx_len, K, k, depth = MID, 45, 12, 5, 3
    tgt, w = make_pair(shape, 4, max_ctx=320, gain_jitter=0.2)
    ctx = ci.uniform_tokens(4, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    kv = co.OracleKV.empty(shape, 320)
    g0 = co.prefill(shape, w, kv, ctx)
    assert tgt.prefill(ctx) == g0
    mask_base, tree_base = ctx_len // 16 * 16, (ctx_len + 15) // 16 * 16
    words = (tree_base + 1 + K * depth - mask_base + 31) // 32
    cache = card.CandidateCache(K=K, max_depth=depth + 1)
    cache.write(0, [g0], [-1], [1.0])
    # oracle state
    o_toks, o_par, o_sig, o_vis = [g0], [-1], np.array([1.0]), [list(range(ctx_len)) + [tree_base]]
    # device state
    d_toks, d_par, d_sig = [g0], [-1], torch.ones(1, dtype=torch.float32, device="cuda:0")
    st, d_rows = card.card_tree_mask_level(None, [-1], tree_base, ctx_len, mask_base, words)
    first, compared = tree_base, 0
    for l in range(depth):
        n = len(o_toks)
        ref = co.forward_tree_rows(shape, w, kv, o_toks, [ctx_len + l] * n, [first + i for i in range(n)], o_vis)
        probs = co.softmax_rows(ref)
        rt, rs, rp = build_level(probs, o_sig, K, k)
        same_inputs = d_toks == o_toks and d_par == o_par
        res = tgt.draft_level(ctx_len, d_toks, [ctx_len + l] * len(d_toks), first, d_rows, mask_base, k)
        ot = torch.empty(K, dtype=torch.int32, device="cuda:0")
        os_ = torch.empty(K, dtype=torch.float32, device="cuda:0")
        op = torch.empty(K, dtype=torch.int32, device="cuda:0")
        cnt = card.card_cache_select(d_sig, res["topk_tokens"], res["topk_probs"], len(d_toks), k, K, ot, os_, op)
        torch.cuda.synchronize()
        assert cnt == min(K, len(d_toks) * k)
        nt, ns, npar = ot[:cnt].tolist(), os_[:cnt].cpu().numpy().astype(np.float64), op[:cnt].tolist()
        assert cache.write(l + 1, nt, npar, ns.tolist()) == card.CARD_OK
        # decisive: every oracle score differs from its neighbours (and from the first one cut) by > 2 %
        pool = sorted((float(probs[i, t]) * float(o_sig[i]) for i in range(n) for t in np.argsort(-probs[i])[:k]), reverse=True)
        cut = pool[: len(rt) + 1]
        decisive = all(cut[j] > 1.02 * cut[j + 1] for j in range(len(cut) - 1))
        if same_inputs and decisive:
            assert nt == rt.tolist() and npar == rp.tolist()
            np.testing.assert_allclose(ns, rs, rtol=5e-3)
            compared += 1
        # next level: oracle
        new_first = first + n
        o_vis = [o_vis[p] + [new_first + i] for i, p in enumerate(rp.tolist())]
        o_toks, o_par, o_sig = rt.tolist(), rp.tolist(), rs
        # next level: device (mask rows from the host helper, scores stay on the device)
        st, d_rows = card.card_tree_mask_level(d_rows, npar, new_first, ctx_len, mask_base, words)
        assert st == card.CARD_OK
        d_toks, d_par, d_sig = nt, npar, os_[:cnt].clone()
        first = new_first
    assert compared >= 1
    assert cache.depth() == depth + 1
    hit, path, score = cache.query(g0, depth + 1)
    assert hit and path[0] == g0 and len(path) == depth + 1


def test_a_wide_level_in_calls_side_by_side_equals_the_calls_one_after_the_other():
    """A level of 100 nodes on four lanes (each call on its own 64 workgroups, workspace and
    stream) gives bit for bit what four calls in a row on the same grid give, and leaves the same
    keys in the cache."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, seed, ctx_len, n, k = MID, 21, 70, 100, 8
    tgt = card.Target(shape, 320, max_r=32, grid_wgs=64)
    load_synthetic_weights(tgt, shape, seed, 0.2)
    tgt.enable_lanes(4)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    tgt.prefill(ctx)
    rng = np.random.default_rng(seed)
    mask_base, first = ctx_len // 16 * 16, 80
    words = (first + 1 + 2 * n - mask_base + 31) // 32
    st, root_row = card.card_tree_mask_level(None, [-1], first, ctx_len, mask_base, words)
    tgt.draft_level(ctx_len, [5], [ctx_len], first, root_row, mask_base, k)
    toks = rng.integers(0, shape.vocab, size=n).tolist()
    out = {}
    for name, base in (("row", first + 1), ("wide", first + 1)):  # the same slots: the same sums in the same order
        st, rows = card.card_tree_mask_level(root_row, [0] * n, base, ctx_len, mask_base, words)
        assert st == card.CARD_OK
        if name == "wide":
            res = tgt.draft_level_wide(ctx_len, toks, [ctx_len + 1] * n, base, rows, mask_base, k)
            tk, tp = res["topk_tokens"].cpu(), res["topk_probs"].cpu()
        else:
            parts = [tgt.draft_level(ctx_len, toks[c:c + 32], [ctx_len + 1] * len(toks[c:c + 32]), base + c, rows[c:c + 32],
                                     mask_base, k) for c in range(0, n, 32)]
            tk = torch.cat([p["topk_tokens"].cpu() for p in parts])
            tp = torch.cat([p["topk_probs"].cpu() for p in parts])
        kk, vv = tgt.kv_gather(shape.n_layers - 1, base, n)
        out[name] = (tk, tp, kk, vv)
    for a, b in zip(out["row"], out["wide"]):
        assert torch.equal(a, b)
    assert (out["wide"][0] >= 0).all()


@pytest.mark.parametrize("n", [8, 13, 29])
def test_a_chain_forwarded_as_tree_rows_equals_the_verify_step_bit_for_bit(n):
    """Tree rows whose mask is the plain causal chain (row i sees the context and rows 0..i, slots
    = positions) are the rows of a verification step: card_draft_level must then give the logits
    and keys of card_verify bit for bit - the tree mask, the separate positions and slots change
    what a row sees, never how its sums are taken."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, seed, ctx_len = MID, 31, 75
    tgt = card.Target(shape, 192, max_r=32)
    load_synthetic_weights(tgt, shape, seed, 0.2)
    toks = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len + n, shape.vocab).tolist()
    tgt.prefill(toks[:ctx_len])
    ref = tgt.verify(ctx_len, -1, toks[ctx_len:], want_logits=True)
    k_ref, v_ref = tgt.kv_gather(shape.n_layers - 1, ctx_len, n)
    mask_base = ctx_len // 16 * 16
    words = (ctx_len + n - mask_base + 31) // 32
    rows, prev = [], None
    for i in range(n):
        st, row = card.card_tree_mask_level(prev, [-1 if i == 0 else 0], ctx_len + i, ctx_len, mask_base, words)
        rows.append(row[0])
        prev = row
    res = tgt.draft_level(ctx_len, toks[ctx_len:], [ctx_len + i for i in range(n)], ctx_len, rows, mask_base, 4, want_logits=True)
    assert torch.equal(res["logits"], ref["logits"])
    k, v = tgt.kv_gather(shape.n_layers - 1, ctx_len, n)
    assert torch.equal(k, k_ref) and torch.equal(v, v_ref)
    # the fused top-k's first entry is the arg-max the verify step reports
    assert res["topk_tokens"][:, 0].tolist() == ref["row_argmax"]
