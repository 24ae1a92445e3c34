"""Parity of the HIP path against stored oracle values (tests/golden/*.json, written by
tests/golden/make_golden.py from the CPU oracle alone): the tiny shape in fp64 and the full
8B-shaped workload of the benchmark (32 layers, context 1024, r = 8) in fp32.

Floating point decides integers here (arg-max, accepted prefix), so:
  * rows whose oracle top-1 / top-2 gap exceeds 0.05 must give the oracle's arg-max bit-exactly;
  * the sampled logits must agree within 2e-2 of the row's largest |logit|;
  * accepted_len / correction_token must follow from the GPU's own row arg-maxes by the
    prefix-accept rule (Target verification: accept while candidate j equals the prediction made
    one position earlier), and equal the oracle's wherever every row that takes part is decisive.
"""
import json
import os

import numpy as np
import pytest
import torch

import card_inputs as ci
from gpu_common import GAP, shuffled_pages

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
LOGIT_TOL = 2e-2
# The stated bar is 2e-2; with the cache precision equal on both sides the path measures 4e-4 to
# 8e-4 at full depth, so a regression shows long before the bar: the full-size cases also hold 4e-3.
LOGIT_TOL_FULL = 4e-3


def _prefix_accept(pending, cand, row_argmax):
    pred = [pending] + list(row_argmax)
    j = 0
    while j < len(cand) and cand[j] == pred[j]:
        j += 1
    return j, pred[j]


def _run(golden_name, logit_tol=LOGIT_TOL):
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    with open(os.path.join(GOLDEN, golden_name)) as f:
        g = json.load(f)
    shape, seed, ctx_len, r = ci.SHAPES[g["shape"]], g["seed"], g["ctx"], g["r"]
    if g.get("layers", shape.n_layers) != shape.n_layers:  # a stored case at reduced depth (the 70B widths)
        shape = shape.with_layers(g["layers"])
    extra = len(g["window"]["extra_ctx"]) if "window" in g else 0
    max_ctx = (ctx_len + extra + 2 * r + 8 + 15) // 16 * 16
    tgt = card.Target(shape, max_ctx, page_order=shuffled_pages(max_ctx // 16, seed))
    load_synthetic_weights(tgt, shape, seed)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    tgt.prefill(ctx)
    g0 = g["greedy"][0]  # the oracle's pending token: both sides judge row 0 against the same token
    idx = g["sample_idx"]
    checked_rows = 0
    for case in g["cases"]:
        cand = case["cand"]
        res = tgt.verify(ctx_len, g0, cand, want_logits=True)
        gpu_arg = res["row_argmax"]
        # integers the path decides: consistent with its own arg-maxes
        assert (res["accepted_len"], res["correction_token"]) == _prefix_accept(g0, cand, gpu_arg), case["j"]
        assert res["kv_first_slot"] == ctx_len and res["kv_count"] == res["accepted_len"]
        decisive = [gap > GAP for gap in case["row_gap"]]
        for m in range(r):
            if decisive[m]:
                assert gpu_arg[m] == case["row_argmax"][m], (case["j"], m, case["row_gap"][m])
                checked_rows += 1
            else:  # a near-tie: either of the oracle's two best tokens
                assert gpu_arg[m] in case["row_top2"][m], (case["j"], m, case["row_gap"][m])
        # rows 0 .. accepted_len - 1 decide the accepted prefix, row accepted_len the correction
        a = case["accepted_len"]
        if all(decisive[: min(a + 1, r)]):
            assert res["accepted_len"] == a and res["correction_token"] == case["correction_token"], case["j"]
        # sampled logits
        got = res["logits"][:, idx].double().numpy()
        ref = np.asarray(case["logit_sample"], dtype=np.float64)
        err = np.abs(got - ref).max(axis=1) / np.asarray(case["row_absmax"])
        assert err.max() <= logit_tol, (case["j"], err.tolist())
        # the row maximum itself (not among the samples unless it is a greedy token)
        full = res["logits"].double().numpy()
        assert np.all(np.abs(np.abs(full).max(axis=1) - np.asarray(case["row_absmax"])) / np.asarray(case["row_absmax"])
                      <= logit_tol)
    assert checked_rows > 0
    # at full size too, a verified row has the plain decode step's logits bit for bit
    cand = g["cases"][-1]["cand"]
    step = tgt.verify(ctx_len, g0, cand, want_logits=True)["logits"]
    if r <= 8:
        for i in range(min(3, r)):
            one = tgt.verify(ctx_len + i, -1, [cand[i]], want_logits=True)["logits"][0]
            assert torch.equal(step[i], one), i
    else:  # (inside the kernel that runs this step length: the shortest step it takes)
        lo = 9 if r <= 16 else 17
        short = tgt.verify(ctx_len, g0, cand[:lo], want_logits=True)["logits"]
        assert torch.equal(step[:lo], short)
    _window_case(tgt, g, ctx, logit_tol)
    return g


def _window_case(tgt, g, ctx, logit_tol):
    """The stored fully decisive step (make_golden.py --window): the context is followed by the
    oracle's own greedy tokens up to a point where r rows in a row have a top-1/top-2 gap above
    0.05; the candidates are the next r greedy tokens, so the step is accepted in full and the
    HIP path has to give accepted_len = r and the oracle's correction token bit-exactly."""
    w = g.get("window")
    if w is None:
        return
    r, n = g["r"], w["ctx_len"]
    assert n == g["ctx"] + len(w["extra_ctx"]) and all(gap > GAP for gap in w["row_gap"])
    assert w["accepted_len"] == r and w["cand"][0] == w["pending"]
    tgt.prefill(list(ctx) + w["extra_ctx"])
    res = tgt.verify(n, w["pending"], w["cand"], want_logits=True)
    assert res["row_argmax"] == w["row_argmax"]
    assert (res["accepted_len"], res["correction_token"]) == (r, w["correction_token"])
    assert (res["kv_first_slot"], res["kv_count"]) == (n, r)
    got = res["logits"][:, w["sample_idx"]].double().numpy()
    ref = np.asarray(w["logit_sample"], dtype=np.float64)
    err = np.abs(got - ref).max(axis=1) / np.asarray(w["row_absmax"])
    assert err.max() <= logit_tol, err.tolist()


def test_tiny_against_stored_oracle_values():
    g = _run("tiny_seed1.json")
    assert g["kv_store"] == "bf16" and "window" in g


FULL = sorted(f for f in os.listdir(GOLDEN) if f.startswith("llama8b_seed") and f.endswith(".json") and "_ctx" not in f)
# full-depth cases at other shapes / context lengths (file name: <shape>_seed<seed>_ctx<N>.json)
OTHER = sorted(f for f in os.listdir(GOLDEN) if f.endswith(".json") and "_seed" in f and f not in FULL
               and not f.endswith("_draft.json") and not f.startswith("tiny"))


@pytest.mark.parametrize("golden_name", FULL)
def test_full_size_workload_against_stored_oracle_values(golden_name):
    """The configuration bench.py times: 8B shape, 1024 tokens of context, r = 8, one workgroup
    per compute unit; planted prefixes j = 0, 4, 8; one case per stored seed."""
    g = _run(golden_name, LOGIT_TOL_FULL)
    assert g["shape"] == "llama8b" and g["ctx"] == 1024 and g["r"] == 8 and g["kv_store"] == "bf16"
    torch.cuda.synchronize()


@pytest.mark.parametrize("golden_name", OTHER)
def test_full_depth_at_other_shapes_and_contexts(golden_name):
    """Full depth where the host oracle can reach it: the Qwen-7B-shaped model (28 layers) and the
    8B shape at a context long enough for many cuts of the page list and in-loop page refills at
    the real widths.  Same bars as the headline workload."""
    g = _run(golden_name, LOGIT_TOL_FULL)
    assert g["kv_store"] == "bf16" and (ci.SHAPES[g["shape"]].n_layers >= 28 or g["shape"] == "llama70b")
    torch.cuda.synchronize()


DRAFT = sorted(f for f in os.listdir(GOLDEN) if f.endswith("_draft.json"))


@pytest.mark.parametrize("golden_name", DRAFT)
def test_draft_tree_forward_at_full_depth(golden_name):
    """card_draft_level on the 1B-shaped draft (16 layers, context 1024) against stored oracle values:
    a tree of 1 + 40 + 24 nodes, the 40-node level in two calls.  Sampled logits within the bar of
    the verify step; the returned top-k set equals the oracle's where the k-th and (k+1)-th oracle
    logits are more than 0.05 apart, rank j holds the oracle's token while every gap down to rank j
    is that large; every returned probability is the softmax value of that token in the path's own logit
    row (5e-3 in the logarithm), whose log-sum-exp lies within the logit bar of the oracle's."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    with open(os.path.join(GOLDEN, golden_name)) as f:
        g = json.load(f)
    shape, seed, ctx_len, k = ci.SHAPES[g["shape"]], g["seed"], g["ctx"], g["k"]
    assert g["kv_store"] == "bf16"
    n_nodes = sum(len(lv["tokens"]) for lv in g["levels"])
    max_ctx = (g["tree_base"] + n_nodes + 8 + 15) // 16 * 16
    tgt = card.Target(shape, max_ctx, max_r=32, page_order=shuffled_pages(max_ctx // 16, seed))
    load_synthetic_weights(tgt, shape, seed)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    g0 = tgt.prefill(ctx)
    idx = g["sample_idx"]
    mask_base = ctx_len // 16 * 16
    words = (g["tree_base"] + n_nodes - mask_base + 31) // 32
    prev_rows, worst, sets, orders = None, 0.0, 0, 0
    for l, lv in enumerate(g["levels"]):
        toks, parents, first = lv["tokens"], lv["parents"], lv["first_slot"]
        st, rows = card.card_tree_mask_level(prev_rows, parents, first, ctx_len, mask_base, words)
        assert st == card.CARD_OK
        for c0 in range(0, len(toks), 32):
            c1 = min(len(toks), c0 + 32)
            res = tgt.draft_level(ctx_len, toks[c0:c1], [lv["position"]] * (c1 - c0), first + c0, rows[c0:c1], mask_base, k,
                                  want_logits=True)
            tk, tp = res["topk_tokens"].cpu().numpy(), res["topk_probs"].cpu().double().numpy()
            for i in range(c0, c1):
                ref = lv["rows"][i]
                got = res["logits"][i - c0].double().numpy()
                err = float(np.abs(got[idx] - np.array(ref["logit_sample"])).max() / ref["absmax"])
                worst = max(worst, err)
                assert err <= LOGIT_TOL_FULL, (l, i, err)
                top, tl = ref["top"], ref["top_logits"]
                mine = tk[i - c0].tolist()
                assert len(set(mine)) == k and all(tp[i - c0][j] >= tp[i - c0][j + 1] for j in range(k - 1))
                # probabilities: the softmax of the path's own logit row (fused online log-sum-exp against the
                # plain one in fp64), and that log-sum-exp within the logit bar of the oracle's
                lse = float(np.log(np.exp(got - got.max()).sum()) + got.max())
                assert abs(lse - ref["lse"]) <= LOGIT_TOL_FULL * ref["absmax"], (l, i)
                for j, t in enumerate(mine):
                    assert abs(np.log(tp[i - c0][j]) - (got[t] - lse)) <= 5e-3, (l, i, j)
                if tl[k - 1] - tl[k] > GAP:
                    assert set(mine) == set(top[:k]), (l, i)
                    sets += 1
                for j in range(k):  # rank j is fixed while every gap down to it is decisive
                    if tl[j] - tl[j + 1] <= GAP:
                        break
                    assert mine[j] == top[j], (l, i, j)
                    orders += 1
        prev_rows = rows
    print(f"[{golden_name}] worst sampled logit error {worst:.2e} of the row maximum; {sets} rows with a decisive top-{k} set, "
          f"{orders} decisive ranks; g0 {'equal' if g0 == g['g0'] else 'differs (near tie)'}")
    assert sets >= 8 and orders >= 40


@pytest.mark.parametrize("ctx_len", [8200, 32700])
def test_long_contexts_at_full_size_hold_what_holds_at_any_size(ctx_len):
    """8B shape at contexts the host oracle cannot reach in reasonable time (many cuts, page-buffer
    refills inside a cut): properties that hold at any size.  (1) A row of an eight-row step has
    the plain decode step's logits bit for bit.  (2) Where the pages lie in the pool does not
    matter: after moving every page to another place (and saying so in the block table) the step
    gives the same bits.  (3) The keys a step stores are the ones a plain decode step stores.
    The cache holds noise for the context (no prefill of 32k tokens needed for any of this)."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, seed, r = ci.SHAPES["llama8b"], 4, 8
    max_ctx = (ctx_len + 64 + 15) // 16 * 16
    n_pages = max_ctx // 16
    tgt = card.Target(shape, max_ctx, page_order=shuffled_pages(n_pages, seed))
    load_synthetic_weights(tgt, shape, seed)
    gen = torch.Generator(device=tgt.device)
    gen.manual_seed(seed)
    for pool in (tgt.k_pages, tgt.v_pages):
        v = pool.view(torch.bfloat16)
        for i in range(0, v.numel(), 1 << 28):
            v[i:i + (1 << 28)].normal_(0.0, 0.5, generator=gen)
    toks = ci.uniform_tokens(seed, "cand_tokens", 0, r, shape.vocab).tolist()
    plain, keys = [], []
    for i in range(r):
        plain.append(tgt.verify(ctx_len + i, -1, [toks[i]], want_logits=True)["logits"][0].clone())
    k_plain, v_plain = tgt.kv_gather(shape.n_layers - 1, ctx_len, r)
    step = tgt.verify(ctx_len, -1, toks, want_logits=True)["logits"].clone()
    for i in range(r):
        assert torch.equal(step[i], plain[i]), i
    k_step, v_step = tgt.kv_gather(shape.n_layers - 1, ctx_len, r)
    assert torch.equal(k_step, k_plain) and torch.equal(v_step, v_plain)
    # move the pages: new place of logical page j = perm[old place]
    old = tgt.block_table.cpu()
    perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(seed + 1))
    per_layer = tgt.k_pages.numel() // shape.n_layers
    for pool in (tgt.k_pages, tgt.v_pages):
        view = pool.view(shape.n_layers, n_pages, per_layer // n_pages)
        moved = torch.empty_like(view)
        moved[:, perm.to(tgt.device)] = view
        view.copy_(moved)
    tgt.block_table.copy_(perm[old.long()].to(torch.int32))
    again = tgt.verify(ctx_len, -1, toks, want_logits=True)["logits"]
    assert torch.equal(again, step)
