#!/usr/bin/env python3
"""Writes the stored expected values of the parity tests.  Calls only the CPU oracle (oracle/) on
the seeded synthetic inputs (card_inputs/); nothing here touches the HIP path.

Usage:
  python tests/golden/make_golden.py llama8b 1 [--r R] [--ctx N] [--window W]
      (full-size shapes: about an hour on 8 cores, 30 GB of host memory)
  python tests/golden/make_golden.py tiny-planted
      (seconds)
  python tests/golden/make_golden.py draft llama1b 1
      (a few minutes)

Per-shape output tests/golden/<shape>_seed<seed>[_ctx<N>].json: the greedy stream g0..g_r of the
oracle after a context of N uniform tokens with each step's top-1/top-2 gap, and for the planted
prefix lengths j = 0, r/2, r the oracle's verify result plus a sample of final-layer logits per
row.  With --window W the oracle decodes W greedy tokens and looks for the first run of r
consecutive rows whose gap exceeds 0.05: a verify step placed there (context = the N uniform tokens
followed by the stream up to that point, candidates = the next r greedy tokens) is accepted in
full and every row that decides it is decisive, so the HIP path has to reproduce accepted_len = r
and the correction token bit-exactly.  That case is stored under "window".

draft writes tests/golden/<shape>_seed<seed>_draft.json: the draft-side tree forward (Cache
Construction, eq. (1)-(2); Mask Construction for Draft Model) at full depth.  Behind a context of
N uniform tokens sits a tree of three levels (the root, 40 nodes, 24 nodes; seeded random tokens
and parents); per node the oracle's k + 1 largest logits with their tokens, the log-sum-exp of the
row, its largest |logit| and a sample of logits.

tiny-planted writes tests/golden/tiny_planted_kept.json: for the small configuration, seeds
1..20 and every planted prefix length j, whether all deciding rows are decisive in the oracle,
i.e. whether the GPU test has to hold the bit-exact assertion for (seed, j).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import card_inputs as ci  # noqa: E402
from oracle import card_oracle as co  # noqa: E402
from oracle.from_inputs import oracle_weights  # noqa: E402

GAP = 0.05
GOLDEN = os.path.join(ROOT, "tests", "golden")


def case_record(res, cand, j, sample_idx):
    top2 = [np.argsort(row)[-2:][::-1].tolist() for row in res.logits]
    return {
        "j": j, "cand": [int(c) for c in cand], "accepted_len": res.accepted_len,
        "correction_token": res.correction_token, "row_argmax": res.row_argmax, "row_gap": res.row_gap,
        "row_top2": top2, "row_absmax": [float(np.abs(row).max()) for row in res.logits],
        "logit_sample": [[float(row[i]) for i in sample_idx] for row in res.logits],
    }


def tiny_planted():
    shape = ci.SHAPES["tiny"]
    kept = {}
    for seed in range(1, 21):
        w = oracle_weights(shape, seed)
        ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
        kv = co.OracleKV.empty(shape, 160)
        g0 = co.prefill(shape, w, kv, ctx)
        greedy, _ = co.greedy_decode_cached(shape, w, kv, shape.ctx, g0, shape.r)
        js = []
        for j in range(shape.r + 1):
            cand = ci.plant_candidates(greedy, j, shape.r, shape.vocab, seed, stream=j)
            res = co.verify(shape, w, kv, shape.ctx, g0, cand)
            assert res.accepted_len == j
            # rows 0..j-2 decide the accepted prefix, row j-1 supplies the correction token
            if all(g > GAP for g in res.row_gap[:j]):
                js.append(j)
        kept[str(seed)] = js
    out = {"shape": "tiny", "ctx": shape.ctx, "r": shape.r, "gap": GAP, "kv_store": "bf16",
           "gain_jitter": 0.0, "kept": kept, "n_kept": sum(len(v) for v in kept.values())}
    path = os.path.join(GOLDEN, "tiny_planted_kept.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, out["n_kept"], "of", 20 * (shape.r + 1))


def draft_golden(name, seed, k=8):
    from oracle.cache_oracle import tree_mask

    shape = ci.SHAPES[name]
    n_ctx = shape.ctx
    dt = np.float32 if shape.d_model >= 2048 else np.float64
    t0 = time.time()
    w = oracle_weights(shape, seed, dtype=dt)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, n_ctx, shape.vocab).tolist()
    widths = [1, 40, 24]
    tree_base = (n_ctx + 15) // 16 * 16
    kv = co.OracleKV.empty(shape, tree_base + sum(widths) + 8, dt)
    g0 = co.prefill(shape, w, kv, ctx, dt, chunk=128)
    print(f"prefill done {time.time() - t0:.0f}s g0={g0}", flush=True)
    rng = np.random.default_rng(seed)
    levels, prev = [], 0
    for l, n in enumerate(widths):
        toks = [int(g0)] if l == 0 else rng.integers(0, shape.vocab, size=n).tolist()
        parents = [-1] * n if l == 0 else rng.integers(0, prev, size=n).tolist()
        levels.append((toks, parents))
        prev = n
    mask = tree_mask([p for _, p in levels])
    offs = np.cumsum([0] + widths)
    sample_idx = sorted(set(np.random.default_rng(1234).integers(0, shape.vocab, size=48).tolist()))
    out_levels = []
    for l, (toks, parents) in enumerate(levels):
        n = len(toks)
        first = tree_base + int(offs[l])
        visible = [list(range(n_ctx)) + [tree_base + int(j) for j in np.flatnonzero(mask[offs[l] + i])] for i in range(n)]
        logits = co.forward_tree_rows(shape, w, kv, toks, [n_ctx + l] * n, [first + i for i in range(n)], visible, dt)
        rows = []
        for row in logits.astype(np.float64):
            order = sorted(range(row.shape[0]), key=lambda t: (-row[t], t))[: k + 1]
            lse = float(np.log(np.exp(row - row.max()).sum()) + row.max())
            rows.append({"top": [int(t) for t in order], "top_logits": [float(row[t]) for t in order], "lse": lse,
                         "absmax": float(np.abs(row).max()), "logit_sample": [float(row[i]) for i in sample_idx]})
        out_levels.append({"tokens": [int(t) for t in toks], "parents": [int(q) for q in parents], "first_slot": first,
                           "position": n_ctx + l, "rows": rows})
        print(f"level {l}: {n} rows {time.time() - t0:.0f}s", flush=True)
    out = {"shape": name, "seed": seed, "ctx": n_ctx, "k": k, "tree_base": tree_base, "oracle_dtype": str(np.dtype(dt)),
           "kv_store": kv.store, "g0": int(g0), "sample_idx": sample_idx, "levels": out_levels}
    path = os.path.join(GOLDEN, f"{name}_seed{seed}_draft.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, f"{time.time() - t0:.0f}s", flush=True)


def main():
    if len(sys.argv) > 1 and sys.argv[1] == "tiny-planted":
        tiny_planted()
        return
    if len(sys.argv) > 3 and sys.argv[1] == "draft":
        draft_golden(sys.argv[2], int(sys.argv[3]))
        return
    ap = argparse.ArgumentParser()
    ap.add_argument("shape")
    ap.add_argument("seed", type=int)
    ap.add_argument("--r", type=int, default=None)
    ap.add_argument("--ctx", type=int, default=None)
    ap.add_argument("--window", type=int, default=0, help="greedy tokens to scan for a fully decisive run of r rows")
    ap.add_argument("--layers", type=int, default=0, help="reduced depth: the first N layers of the shape (for widths whose "
                    "full depth does not fit the host: the 70B shape)")
    ap.add_argument("--chunk", type=int, default=128, help="rows per oracle forward call while the context is prefilled "
                    "(the rows of a call are independent of how the context is cut; larger pieces only spread the "
                    "per-call cost of widening the weights over more rows)")
    args = ap.parse_args()
    name, seed = args.shape, args.seed
    shape = ci.SHAPES[name]
    r = shape.r if args.r is None else args.r
    n_ctx = shape.ctx if args.ctx is None else args.ctx
    if args.layers:
        shape = shape.with_layers(args.layers)
    dt = np.float32 if shape.d_model >= 2048 else np.float64
    t0 = time.time()
    w = oracle_weights(shape, seed, dtype=dt)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, n_ctx, shape.vocab).tolist()
    n_new = max(r, args.window)
    kv = co.OracleKV.empty(shape, n_ctx + n_new + r + 8, dt)
    # (co.prefill's own loop, written out so that a long context reports its progress)
    for s0 in range(0, n_ctx, args.chunk):
        last = co.forward_rows(shape, w, kv, ctx[s0: s0 + args.chunk], s0, dt)
        print(f"prefilled {min(n_ctx, s0 + args.chunk)} of {n_ctx} {time.time() - t0:.0f}s", flush=True)
    g0 = int(co.argmax_lowest(last[-1]))
    print(f"prefill done {time.time() - t0:.0f}s g0={g0}", flush=True)
    # decode in pieces of r tokens and stop at the first fully decisive run of r rows
    greedy, gaps = [g0], []
    while len(gaps) < n_new:
        more, mg = co.greedy_decode_cached(shape, w, kv, n_ctx + len(gaps), greedy[-1], min(r, n_new - len(gaps)), dt)
        greedy += more[1:]
        gaps += mg
        if args.window and len(gaps) >= r and any(all(g > GAP for g in gaps[k: k + r]) for k in range(len(gaps) - r + 1)):
            break
    n_new = len(gaps)
    print(f"greedy {greedy} gaps {gaps} {time.time() - t0:.0f}s", flush=True)
    rng = np.random.default_rng(1234)
    sample_idx = sorted(set(rng.integers(0, shape.vocab, size=48).tolist() + [int(t) for t in greedy[: r + 1]]))
    out = {"shape": name, "seed": seed, "ctx": n_ctx, "r": r, "oracle_dtype": str(np.dtype(dt)), "kv_store": kv.store,
           "prefill_chunk": args.chunk, "layers": shape.n_layers,
           "greedy": [int(g) for g in greedy[: r + 1]], "greedy_gaps": [float(g) for g in gaps[:r]],
           "sample_idx": sample_idx}

    if args.window:
        # gaps[i] belongs to the row fed greedy[i] at position n_ctx + i; a step at offset k feeds
        # greedy[k .. k+r): rows k .. k+r-1 decide it (the last one supplies the correction token)
        k = next((k for k in range(0, n_new - r + 1) if all(g > GAP for g in gaps[k: k + r])), None)
        print(f"window scan over {n_new} greedy tokens: offset {k}", flush=True)
        out["window_scanned"] = n_new
        if k is not None:
            cand = [int(t) for t in greedy[k: k + r]]
            # the cache already holds the stream's keys up to n_ctx + n_new: the step rewrites
            # rows n_ctx + k .. with the same tokens
            res = co.verify(shape, w, kv, n_ctx + k, greedy[k], cand, dt, keep_logits=True)
            assert res.accepted_len == r and res.correction_token == greedy[k + r], (res.accepted_len, k)
            assert all(g > GAP for g in res.row_gap)
            widx = sorted(set(sample_idx + cand + [int(greedy[k + r])]))
            rec = case_record(res, cand, r, widx)
            rec.update({"offset": k, "ctx_len": n_ctx + k, "extra_ctx": [int(t) for t in greedy[:k]],
                        "pending": int(greedy[k]), "sample_idx": widx})
            out["window"] = rec
            print(f"window case at ctx {n_ctx + k}: accepted {res.accepted_len}, gaps {res.row_gap} "
                  f"{time.time() - t0:.0f}s", flush=True)
            # verify has just rewritten rows n_ctx+k .. n_ctx+k+r-1 with the same tokens: the cache
            # is unchanged for the cases below

    cases = []
    for j in sorted({0, r // 2, r}):
        cand = ci.plant_candidates(greedy, j, r, shape.vocab, seed, stream=j)
        res = co.verify(shape, w, kv, n_ctx, g0, cand, dt, keep_logits=True)
        cases.append(case_record(res, cand, j, sample_idx))
        print(f"case j={j} accepted {res.accepted_len} {time.time() - t0:.0f}s", flush=True)
    out["cases"] = cases
    suffix = ("" if n_ctx == ci.SHAPES[name].ctx else f"_ctx{n_ctx}") + (f"_L{args.layers}" if args.layers else "")
    path = os.path.join(GOLDEN, f"{name}_seed{seed}{suffix}.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, f"{time.time() - t0:.0f}s", flush=True)


if __name__ == "__main__":
    main()
