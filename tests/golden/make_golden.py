#!/usr/bin/env python3
"""Writes the stored expected values of the full-size parity test.  Calls only the CPU oracle
(oracle/) on the seeded synthetic inputs (card_inputs/); nothing here touches the HIP path.

Usage: python tests/golden/make_golden.py llama8b 1 [r]      (about half an hour on 8 cores)

Output tests/golden/<shape>_seed<seed>.json: the greedy stream g0..g_r of the oracle after a
context of `shape.ctx` uniform tokens with each step's top-1/top-2 gap, and for a few planted
prefix lengths j the oracle's verify result plus a sample of final-layer logits per row.
"""
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


def main():
    name, seed = sys.argv[1], int(sys.argv[2])
    shape = ci.SHAPES[name]
    r = int(sys.argv[3]) if len(sys.argv) > 3 else shape.r
    dt = np.float32 if shape.d_model >= 2048 else np.float64
    t0 = time.time()
    w = oracle_weights(shape, seed, dtype=dt)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    kv = co.OracleKV.empty(shape, shape.ctx + 2 * r + 8, dt)
    g0 = co.prefill(shape, w, kv, ctx, dt, chunk=128)
    print(f"prefill done {time.time() - t0:.0f}s g0={g0}", flush=True)
    greedy, gaps = co.greedy_decode_cached(shape, w, kv, shape.ctx, g0, r, dt)
    print(f"greedy {greedy} gaps {gaps} {time.time() - t0:.0f}s", flush=True)
    rng = np.random.default_rng(1234)
    sample_idx = sorted(set(rng.integers(0, shape.vocab, size=48).tolist() + [int(t) for t in greedy]))
    cases = []
    for j in sorted({0, r // 2, r}):
        cand = ci.plant_candidates(greedy, j, r, shape.vocab, seed, stream=j)
        res = co.verify(shape, w, kv, shape.ctx, g0, cand, dt, keep_logits=True)
        top2 = [np.argsort(row)[-2:][::-1].tolist() for row in res.logits]
        cases.append({
            "j": j, "cand": [int(c) for c in cand], "accepted_len": res.accepted_len,
            "correction_token": res.correction_token, "row_argmax": res.row_argmax, "row_gap": res.row_gap,
            "row_top2": top2, "row_absmax": [float(np.abs(row).max()) for row in res.logits],
            "logit_sample": [[float(row[i]) for i in sample_idx] for row in res.logits],
        })
        print(f"case j={j} accepted {res.accepted_len} {time.time() - t0:.0f}s", flush=True)
    out = {"shape": name, "seed": seed, "ctx": shape.ctx, "r": r, "oracle_dtype": str(np.dtype(dt)), "kv_store": kv.store,
           "greedy": [int(g) for g in greedy], "greedy_gaps": [float(g) for g in gaps],
           "sample_idx": sample_idx, "cases": cases}
    path = os.path.join(ROOT, "tests", "golden", f"{name}_seed{seed}.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, f"{time.time() - t0:.0f}s", flush=True)


if __name__ == "__main__":
    main()
