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
OTHER = sorted(f for f in os.listdir(GOLDEN) if "_ctx" in f and f.endswith(".json"))


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
    assert g["kv_store"] == "bf16" and ci.SHAPES[g["shape"]].n_layers >= 28
    torch.cuda.synchronize()
