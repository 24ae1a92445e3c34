#!/usr/bin/env python3
"""Benchmark of the CARD verify step on one MI355X.

A step is one card_verify call: r = 8 candidates forwarded through the 8B-shaped decoder
(32 layers, d 4096, 32/8 heads of 128, FFN 14336, vocab 128256) against 1024 tokens of paged
bf16 KV cache, then arg-max / prefix-accept / correction.  Weights, KV cache and candidate
tokens are resident in HBM before the timed region starts.  Candidates follow the planted-prefix
recipe (first j tokens are the target's own greedy tokens, j cycling over 0..8).

Prints ONE JSON line: verified tokens/s (value), latency, the HBM roofline of the dominant
kernel measured with HIP events inside this run, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# the paper's end-to-end speedups are for other hardware and another metric: context only
PAPER_CONTEXT = "CARD paper: up to 4.83x over autoregressive decoding on 3x A800-80GB, HF Transformers 4.31"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--shape", default="llama8b")
    ap.add_argument("--ctx", type=int, default=None)
    ap.add_argument("--r", type=int, default=None)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a 1 GiB device copy (calibration) and 5 verify steps, no timing")
    return ap.parse_args()


def step_bytes(shape, ctx: int) -> int:
    """Algorithmic HBM bytes of one verify step = one launch of the verify kernel: every bf16
    weight of the layers and of the vocabulary head read once, plus the bf16 K and V of the
    context read once (activations and the r new KV rows are below 0.1 % and left out)."""
    return shape.streamed_weight_bytes() + shape.kv_bytes(ctx)


def cpu_baseline(shape, seed: int, ctx: int, r: int, cand):
    """The oracle as it stands, timed on the host: verify steps of the 2-layer and 4-layer
    truncations of the workload (same widths, same context, vocabulary head included), fp32,
    median of 10 after one warm-up (about 10 s of CPU work); the full-depth time is extrapolated
    linearly in depth and labelled as such."""
    import numpy as np
    from oracle import card_oracle as co
    from oracle.from_inputs import oracle_weights

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    import card_inputs as ci
    import torch

    s2 = shape.with_layers(4)
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    w = oracle_weights(s2, seed, dtype=np.float32, device=dev)
    ctx_tokens = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx, shape.vocab).tolist()
    kv = co.OracleKV.empty(s2, ctx + r, np.float32)
    t0 = time.time()
    co.prefill(s2, w, kv, ctx_tokens, np.float32, chunk=128)
    t_prefill = time.time() - t0

    def timed(cfg):
        ts = []
        for i in range(11):
            t = time.time()
            co.verify(cfg, w, kv, ctx, -1, cand, np.float32)
            ts.append(time.time() - t)
        return statistics.median(ts[1:])

    t2 = timed(s2)
    t1 = timed(shape.with_layers(2))
    per_layer = max(t2 - t1, 0.0) / 2
    t_full = t1 + (shape.n_layers - 2) * per_layer
    return {
        "value": r / t_full,
        "unit": "tokens/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": (f"oracle verify step (fp32 numpy, r={r}, ctx={ctx}), median of 10 at depth 2 ({t1:.3f} s) and "
                   f"depth 4 ({t2:.3f} s) of {shape.n_layers}, same widths and vocabulary head; "
                   f"full depth extrapolated linearly to {t_full:.2f} s; untimed oracle prefill {t_prefill:.1f} s"),
    }


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the verify step on ONE GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import card_inputs as ci
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape = ci.SHAPES[args.shape]
    ctx = shape.ctx if args.ctx is None else args.ctx
    r = shape.r if args.r is None else args.r
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    tgt = card.Target(shape, ctx + 64, max_r=32)
    load_synthetic_weights(tgt, shape, args.seed)
    ctx_tokens = ci.uniform_tokens(args.seed, "ctx_tokens", 0, ctx, shape.vocab).tolist()
    g0 = tgt.prefill(ctx_tokens)
    # the target's own greedy continuation (plain decode steps, r = 1) to plant prefixes from
    greedy, n = [g0], ctx
    for _ in range(r):
        res = tgt.verify(n, greedy[-1], [greedy[-1]])
        greedy.append(res["correction_token"])
        n += 1
    cands = [ci.plant_candidates(greedy, j, r, shape.vocab, args.seed, stream=j) for j in range(r + 1)]
    cand_dev = torch.tensor(cands, dtype=torch.int32, device=dev)
    # planted-prefix invariant on the path being timed
    for j in range(r + 1):
        res = tgt.verify(ctx, g0, cands[j])
        if res["accepted_len"] != j or res["correction_token"] != greedy[j]:
            print(f"bench.py: planted prefix {j} gave {res}", file=sys.stderr)
            sys.exit(1)

    def step(i):
        st = tgt.enqueue_verify(ctx, g0, r, cand=cand_dev[i % (r + 1)])
        if st != card.CARD_OK:
            raise card.CardError(st, "card_verify")

    if args.pmc_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        for i in range(5):
            step(i)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes": 1 << 30, "verify_steps": 5}))
        return

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # roofline of the dominant kernel.  The whole step is ONE kernel (k_verify), so its launch
    # duration is measured with a HIP event pair around every launch, recorded by the library on
    # the stream the kernel is launched on, over a second pass of the same loop.
    n_prof = min(args.steps, 100)
    card.card_profile_enable(n_prof)
    for i in range(n_prof):
        step(i)
    torch.cuda.synchronize()
    st, ms_each = card.card_profile_collect(n_prof)
    kbytes = step_bytes(shape, ctx)
    k_ms = sum(ms_each) / max(len(ms_each), 1)
    achieved = kbytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{args.shape}:ctx{ctx}:r{r}")
        except Exception:
            traffic = None

    out = {
        "metric": "verified_tokens_per_s",
        "value": r / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "verify_latency_us": ms_per_step * 1e3,
        "verify_latency_us_median_launch": statistics.median(ms_each) * 1e3 if ms_each else None,
        # planted j cycles uniformly over 0..r: mean accepted length r/2 (asserted per j above)
        "accepted_tokens_per_s": (r / 2) / (ms_per_step * 1e-3),
        "hbm_fraction_whole_step": kbytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes_per_step": kbytes,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.shape} verify step, ctx {ctx}, r {r}, planted prefix j cycling 0..{r}",
                   "global_batch": 1, "seq_len": ctx, "r": r, "parallelism": "single GPU"},
        "roofline": {"bound": "hbm", "kernel": "k_verify (whole step, one persistent kernel)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": kbytes, "avg_launch_us": k_ms * 1e3, "launches_timed": len(ms_each)},
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, args.seed, ctx, r, cands[r])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
