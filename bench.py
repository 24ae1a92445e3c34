#!/usr/bin/env python3
"""Benchmark of the CARD verify step on one MI355X.

A step is one card_verify call: r = 8 candidates forwarded through the 8B-shaped decoder
(32 layers, d 4096, 32/8 heads of 128, FFN 14336, vocab 128256) against 1024 tokens of paged
bf16 KV cache, then arg-max / prefix-accept / correction.  Weights, KV cache and candidate
tokens are resident in HBM before the timed region starts.  Candidates follow the planted-prefix
recipe (first j tokens are the target's own greedy tokens, j cycling over 0..8).

Prints ONE JSON line: verified tokens/s (value), latency, the HBM roofline of the dominant
kernel measured with HIP events inside this run, the CPU oracle timed on a bounded sample, and
a `sweep` array with the other synthetic configurations (context lengths 512..32768 on the 8B
shape, the 70B shape at r 4/8/16, the Qwen-7B shape at r 1..32 and its query / verify / correct
loop against the shared cache at planted acceptance rates 0.3 / 0.6 / 0.9), each with latency,
tokens/s and the fraction of the HBM roofline.
"""
from __future__ import annotations

import argparse
import gc
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
PREFILL_MAX_CTX = 32768  # contexts beyond this would be perf-only points with noise in the cache pages


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
    ap.add_argument("--sweep", choices=["full", "quick", "none"], default="full",
                    help="full: every synthetic configuration; quick: one point per kind on the headline shape; none")
    ap.add_argument("--draft-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: three cache levels of K = 100 nodes on the 1B-shaped draft, no timing")
    ap.add_argument("--loop-probe", action="store_true",
                    help="for rocprofv3 --kernel-trace runs: the concurrent draft/target loop alone (70B + 1B shapes)")
    ap.add_argument("--timeline", type=int, default=None, metavar="LAYER",
                    help="the kernel's own phase timeline (100 MHz time stamps per workgroup) of one decoder layer of one "
                         "verify step of the workload: medians over the workgroups, no timing of the step")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a 1 GiB device copy (calibration) and 5 verify steps, no timing")
    return ap.parse_args()


def phase_timeline(rig, ctx, r, cand, layer):
    """One verify step with the library's timeline hook on decoder layer `layer`: per workgroup the
    consumer wavefront 0 stamps the phase boundaries (card_profile_timeline).  Reported: per phase
    the median over the workgroups of (this boundary - the previous one), in microseconds, and the
    spread of each boundary (latest - earliest workgroup); the attention figures over the
    workgroups that had an attention task."""
    import numpy as np
    import torch

    import paper_2508_04462_amd as card

    tgt = rig.tgt
    for _ in range(5):
        assert tgt.enqueue_verify(ctx, rig.g0, r, cand=cand) == card.CARD_OK
    torch.cuda.synchronize()
    ts = torch.zeros(256 * 32, dtype=torch.int64, device=tgt.device)
    card.card_profile_timeline(ts, layer)
    assert tgt.enqueue_verify(ctx, rig.g0, r, cand=cand) == card.CARD_OK
    torch.cuda.synchronize()
    card.card_profile_timeline(None, 0)
    t = ts.cpu().numpy().reshape(256, 32).astype(np.float64) * 0.01  # microseconds
    live = t[:, 0] > 0
    t = t[live]
    names = ["qkv", "barrier_after_qkv", "attention", "barrier_after_attention", "o_proj", "barrier_after_o_proj",
             "gate_up", "barrier_after_gate_up", "down", "barrier_after_down"]
    out = {"workgroups": int(live.sum()), "layer": layer, "unit": "us", "phases": {}, "boundary_spread": {}}
    for i, n in enumerate(names):
        out["phases"][n] = round(float(np.median(t[:, i + 1] - t[:, i])), 2)
        out["boundary_spread"][n] = round(float(t[:, i + 1].max() - t[:, i + 1].min()), 2)
    out["layer_total"] = round(float(np.median(t[:, 10] - t[:, 0])), 2)
    for tag, s0 in (("qkv", 21), ("o_proj", 24), ("down", 27)):
        d = {"first_activations_after": round(float(np.median(t[:, s0] - t[:, {21: 0, 24: 4, 27: 8}[s0]])), 2),
             "k_loop": round(float(np.median(t[:, s0 + 1] - t[:, s0])), 2)}
        if s0 != 27:
            d["of_which_waiting_for_fragments"] = round(float(np.median(t[:, s0 + 2])), 2)
        d["reduction_and_epilogue"] = round(float(np.median(t[:, {21: 1, 24: 5, 27: 9}[s0]] - t[:, s0 + 1])), 2)
        if s0 == 21:  # between the k-loop and the reduction the loads of the old context's pages are issued
            d["of_which_page_preload_issue"] = round(float(np.median(t[:, 16] - t[:, 11])), 2)
            d["stores_acknowledged_after"] = round(float(np.median(t[:, 12] - t[:, 1])), 2)
        out[tag + "_detail"] = d
    att = t[t[:, 13] > 0]
    if len(att):
        out["attention_detail"] = {
            "workgroups_with_a_task": int(len(att)),
            "barrier_to_page_loop": round(float(np.median(att[:, 13] - att[:, 2])), 2),
            "page_loop": round(float(np.median(att[:, 14] - att[:, 13])), 2),
            "wavefronts_merged_after": round(float(np.median(att[:, 15] - att[:, 14])), 2),
            "task_done_median": round(float(np.median(att[:, 3] - att[:, 2])), 2),
            "last_merging_workgroup_done_after_barrier": round(float(att[:, 3].max() - np.median(att[:, 2])), 2)}
    return {"timeline": out, "workload": f"{rig.shape.name} ctx {ctx} r {r}"}


def step_bytes(shape, ctx: int) -> int:
    """Algorithmic HBM bytes of one verify step = one launch of the verify kernel: every bf16
    weight of the layers and of the vocabulary head read once, plus the bf16 K and V of the
    context read once (activations and the r new KV rows are below 0.1 % and left out)."""
    return shape.streamed_weight_bytes() + shape.kv_bytes(ctx)


def cpu_baseline(shape, seed: int, ctx: int, r: int, cand):
    """The oracle as it stands, timed on the host at FULL depth: one verify step of the workload
    (fp32 numpy, r rows against a cache of ctx positions), median of 3 after one warm-up.  The
    cache holds zeros instead of a prefilled context (an oracle prefill of 1024 tokens takes half
    an hour; the step's arithmetic and memory traffic do not depend on the cached values).  If the
    host cannot hold the fp32 weights the 2- and 4-layer truncations are timed instead and the
    full depth is extrapolated linearly, labelled as such."""
    import numpy as np
    import torch

    from oracle import card_oracle as co
    from oracle.from_inputs import oracle_weights

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"

    def timed(cfg, w, kv, n):
        ts = []
        for _ in range(n + 1):
            t = time.time()
            co.verify(cfg, w, kv, ctx, -1, cand, np.float32)
            ts.append(time.time() - t)
        return statistics.median(ts[1:]), ts[0]

    need = 4 * (shape.n_layers * shape.weight_elems_per_layer() + 2 * shape.vocab * shape.d_model)
    try:
        avail = os.sysconf("SC_AVPHYS_PAGES") * os.sysconf("SC_PAGE_SIZE")
    except (ValueError, OSError):
        avail = 0
    if avail > 1.6 * need:
        t0 = time.time()
        w = oracle_weights(shape, seed, dtype=np.float32, device=dev)
        kv = co.OracleKV.empty(shape, ctx + r, np.float32)
        t_step, t_first = timed(shape, w, kv, 3)
        return {
            "value": r / t_step, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": (f"oracle verify step at full depth ({shape.n_layers} layers, fp32 numpy, r={r}, ctx={ctx}), median of 3 "
                       f"= {t_step:.2f} s after one warm-up call ({t_first:.1f} s incl. generating the weights); the cache "
                       f"holds zeros, not a prefilled context (timing does not depend on the values); {time.time() - t0:.0f} s in all"),
        }
    s4 = shape.with_layers(4)
    w = oracle_weights(s4, seed, dtype=np.float32, device=dev)
    kv = co.OracleKV.empty(s4, ctx + r, np.float32)
    t4, _ = timed(s4, w, kv, 10)
    t2, _ = timed(shape.with_layers(2), w, kv, 10)
    per_layer = max(t4 - t2, 0.0) / 2
    t_full = t2 + (shape.n_layers - 2) * per_layer
    return {
        "value": r / t_full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"oracle verify step (fp32 numpy, r={r}, ctx={ctx}), median of 10 at depth 2 ({t2:.3f} s) and "
                   f"depth 4 ({t4:.3f} s) of {shape.n_layers}, same widths and vocabulary head; EXTRAPOLATED linearly "
                   f"to full depth: {t_full:.2f} s (host memory too small for the fp32 weights)"),
    }


class Rig:
    """A target model of one shape with its weights, and the pieces the timed loops need."""

    def __init__(self, shape, seed, max_ctx):
        import torch

        import paper_2508_04462_amd as card
        from paper_2508_04462_amd.synthetic import load_synthetic_weights

        self.card, self.torch = card, torch
        self.shape, self.seed = shape, seed
        self.tgt = card.Target(shape, max_ctx + 64, max_r=32)
        load_synthetic_weights(self.tgt, shape, seed)
        self.ctx = None
        self.g0 = None

    def set_context(self, ctx):
        """Cache contents for a context of `ctx` tokens: prefilled from seeded uniform tokens through
        the library up to PREFILL_MAX_CTX, noise pages beyond (perf-only points).  Returns the kind."""
        import card_inputs as ci

        torch, tgt = self.torch, self.tgt
        self.ctx = ctx
        if ctx <= PREFILL_MAX_CTX:
            toks = ci.uniform_tokens(self.seed, "ctx_tokens", 0, ctx, self.shape.vocab).tolist()
            self.g0 = tgt.prefill(toks)
            return "prefilled"
        g = torch.Generator(device=tgt.device)
        g.manual_seed(self.seed)
        for pool in (tgt.k_pages, tgt.v_pages):
            v = pool.view(torch.bfloat16)
            for i in range(0, v.numel(), 1 << 28):
                v[i:i + (1 << 28)].normal_(0.0, 0.5, generator=g)
        self.g0 = 1
        return "noise"

    def greedy(self, n):
        """The target's own greedy continuation g0 .. g_n (plain decode steps, r = 1)."""
        out, pos = [self.g0], self.ctx
        for _ in range(n):
            res = self.tgt.verify(pos, out[-1], [out[-1]])
            out.append(res["correction_token"])
            pos += 1
        return out

    def planted(self, r):
        """Planted-prefix candidates for every j in 0..r, checked on the path that is timed."""
        import card_inputs as ci

        greedy = self.greedy(r)
        cands = [ci.plant_candidates(greedy, j, r, self.shape.vocab, self.seed, stream=j) for j in range(r + 1)]
        for j in range(r + 1):
            res = self.tgt.verify(self.ctx, self.g0, cands[j])
            if res["accepted_len"] != j or res["correction_token"] != greedy[j]:
                raise RuntimeError(f"planted prefix {j} gave {res}")
        return cands

    def time_steps(self, r, cand_dev, steps, warmup, n_prof):
        """(wall ms per step over `steps` calls, [kernel ms of n_prof further launches])."""
        torch, card, tgt = self.torch, self.card, self.tgt
        n = cand_dev.shape[0]

        def step(i):
            st = tgt.enqueue_verify(self.ctx, self.g0, r, cand=cand_dev[i % n])
            if st != card.CARD_OK:
                raise card.CardError(st, "card_verify")

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        # the whole step is ONE kernel: its launch duration comes from a HIP event pair recorded by
        # the library around every launch, on the stream the kernel is launched on
        card.card_profile_enable(n_prof)
        for i in range(n_prof):
            step(i)
        torch.cuda.synchronize()
        _, ms_each = card.card_profile_collect(n_prof)
        return ms, ms_each

    def close(self):
        self.tgt = None
        gc.collect()
        self.torch.cuda.empty_cache()


def sweep_point(rig, r, steps, kv_kind, planted=True):
    torch, shape = rig.torch, rig.shape
    import card_inputs as ci

    cands = None
    if planted and kv_kind == "prefilled":
        try:
            cands = rig.planted(r)
            cand_note = f"planted prefix j cycling 0..{r}"
        except RuntimeError as e:  # a near-tie between the r = 1 decode steps and the r-row step
            cand_note = f"uniform candidates ({e})"
    else:
        cand_note = "uniform candidates"
    if cands is None:
        cands = [ci.uniform_tokens(rig.seed, "cand_tokens", j, r, shape.vocab).tolist() for j in range(4)]
    cand_dev = torch.tensor(cands, dtype=torch.int32, device=rig.tgt.device)
    ms, ms_each = rig.time_steps(r, cand_dev, steps, max(3, steps // 4), steps)
    k_ms = sum(ms_each) / len(ms_each)
    byts = step_bytes(shape, rig.ctx)
    return {"shape": shape.name, "ctx": rig.ctx, "r": r, "kv": kv_kind, "candidates": cand_note, "steps": steps,
            "ms_per_step": ms, "kernel_ms": k_ms, "verified_tokens_per_s": r / (ms * 1e-3),
            "hbm_frac": byts / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes": byts}


def cache_loop(rig, r, p, n_tokens, K=50, width=10):
    """Query / verify / correct against the shared candidate cache (host object of the library) with
    a scripted draft: per position the best path holds the target's own greedy token with
    probability p (independent draws, so the accepted length is truncated-geometric), K nodes per
    level, depth r.  Every step waits for its result: the next query needs the verified tokens.
    Returns accepted tokens/s over the loop (cache writes, query, step, correction all inside)."""
    import numpy as np

    card, tgt, shape = rig.card, rig.tgt, rig.shape
    truth = rig.greedy(n_tokens + r + 1)
    rng = np.random.default_rng(rig.seed)
    cache = card.CandidateCache(K=K, max_depth=r)

    def draft(e):
        cache.write(0, [truth[e]], [-1], [1.0])
        alive, prev = True, 1
        for i in range(1, r):
            right = truth[e + i]
            good = alive and rng.random() < p
            n = K if i > 1 else min(K, width)
            toks = [(right + 1 + k) % shape.vocab for k in range(n)]
            if good:
                toks[0] = right
            elif alive and rng.random() < 0.5:
                toks[1] = right  # the right token sits on a lower-scored sibling
            parents = [0] * min(n, width) + [int(rng.integers(0, prev)) for _ in range(n - min(n, width))]
            scores = [0.9 ** i] + [0.5 ** i * 0.98 ** k for k in range(1, n)]
            cache.write(i, toks, parents, scores)
            alive, prev = good, n

    pos, pending, emitted, steps, hits, left_at = rig.ctx, truth[0], 0, 0, 0, None
    rig.torch.cuda.synchronize()
    t0 = time.perf_counter()
    while emitted < n_tokens:
        draft(emitted)
        hit, path, _ = cache.query(pending, r)
        cand = path if hit else [pending]
        hits += int(hit)
        res = tgt.verify(pos, pending, cand)
        a = res["accepted_len"]
        if a < 1 or res["correction_token"] != truth[emitted + a]:
            # a near-tie decided differently by the r = 1 steps that wrote `truth`: stop here
            left_at = emitted
            break
        cache.correct(cand[:a])
        pos += res["kv_count"]
        pending = res["correction_token"]
        emitted += a
        steps += 1
    dt = time.perf_counter() - t0
    if steps == 0:
        return {"shape": shape.name, "ctx": rig.ctx, "r": r, "kind": "cache_loop", "planted_acceptance": p,
                "error": "the first step already left the greedy text (near-tie)"}
    return {"shape": shape.name, "ctx": rig.ctx, "r": r, "kind": "cache_loop", "planted_acceptance": p, "K": K,
            "left_greedy_text_at": left_at, "steps": steps, "hit_rate": hits / steps, "mean_accepted_len": emitted / steps,
            "ms_per_step": dt * 1e3 / steps, "accepted_tokens_per_s": emitted / dt,
            "plain_decode_tokens_per_s": None}


def concurrent_loop_entries(args, decode_tps, quick, grids=(192, 64)):
    """Draft and target running at the same time on one GPU (two host threads, two streams, the
    compute units split between the two persistent kernels): the paper's own pairing, a 70B-shaped
    target (on 192 workgroups) with a 1B-shaped draft (on 64), context 1024, K = 8 nodes per
    level, top-8 per node, the draft up to twelve levels ahead of the token verified last, the
    target verifying up to eight tokens per step; the draft's agreement with the target is planted
    (random-init models never agree).  Accepted tokens/s of the loop beside the target's plain
    decode rate on the whole GPU: the synthetic form of the paper's speedup over autoregressive
    decoding."""
    import card_inputs as ci
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    t_shape = ci.SHAPES["tiny" if quick else "llama70b"]
    d_shape = ci.ModelShape("tiny-draft", 1, 128, 2, 1, 64, 344, 1024) if quick else ci.SHAPES["llama1b"]
    ctx_len, n_tok = (128, 24) if quick else (1024, 64)
    depth, r_max = (3, 4) if quick else (12, 8)
    # (planted agreement, sibling catch, nodes per cache level; 50 is the paper's smaller cache size)
    runs = ((0.6, 0.0, 8),) if quick else ((0.3, 0.0, 8), (0.6, 0.0, 8), (0.9, 0.0, 8), (0.6, 0.6, 8), (0.9, 0.0, 50))
    n_text = len(runs) * (n_tok + 60) + 24  # room to step over positions where the target's two best tokens nearly tie
    tgt = card.Target(t_shape, ctx_len + n_text + 64, grid_wgs=grids[0])
    load_synthetic_weights(tgt, t_shape, args.seed)
    dr = card.Target(d_shape, ctx_len + n_text + (256 if quick else 1024) + 64, grid_wgs=grids[1])
    load_synthetic_weights(dr, d_shape, args.seed + 100)
    ctx = ci.uniform_tokens(args.seed, "ctx_tokens", 0, ctx_len, t_shape.vocab).tolist()
    g0 = tgt.prefill(ctx)
    dr.prefill(ctx)
    # The target's own text, token by token, with the gap between its two largest logits at every
    # position: where that gap is tiny the arg-max depends on how the rows are cut into steps (the
    # fp32 sums are ordered differently), the loop may emit the other token and everything planted
    # behind it is void.  Runs are placed on stretches without such positions.
    own, gaps, pos = [g0], [], ctx_len
    for _ in range(n_text):
        res = tgt.verify(pos, own[-1], [own[-1]], want_logits=True)
        top2 = res["logits"][0].topk(2).values
        gaps.append(float(top2[0] - top2[1]))  # gaps[i]: of the row that predicts text index i + 1
        own.append(res["correction_token"])
        pos += 1
    tie = 0.0025  # (logits of about 7.5: differences of the summation order reach 0.001-0.002)
    out = []
    n_done = 0
    for p, q, K in runs:
        # each run continues the text behind the previous one, stepping over near ties
        span = n_tok + r_max + 2
        start = n_done
        while n_done + span < n_text and min(gaps[n_done: n_done + span]) < tie:
            n_done += 1 + next(i for i, g in enumerate(gaps[n_done: n_done + span]) if g < tie)
        # the previous run's last steps left rejected candidates in the cache slots behind its end:
        # the stretch that is stepped over is decoded again
        for i in range(start, n_done):
            tgt.verify(ctx_len + i, own[i], [own[i]])
        loop = card.ConcurrentLoop(tgt, dr, ctx_len + n_done, own[n_done], K=K, k=8, depth=depth, r_max=r_max,
                                   plant=card.PlantedAgreement(own[n_done:], p, args.seed, t_shape.vocab, q=q))
        loop.d_ctx = ctx_len
        loop.committed = own[:n_done]
        loop.d_absorbed = 0
        e = {"kind": "concurrent_loop", "target": t_shape.name, "draft": d_shape.name, "ctx": ctx_len + n_done,
             "target_workgroups": grids[0], "draft_workgroups": grids[1], "planted_acceptance": p, "planted_sibling_catch": q,
             "K": K, "k": 8, "depth": depth, "r_max": r_max, "plain_decode_tokens_per_s_whole_gpu": decode_tps,
             "smallest_top2_gap_of_the_stretch": min(gaps[n_done: n_done + n_tok + r_max + 2])}
        try:
            res = loop.run(n_tok)
            em, tr = loop.emitted[: n_tok + 1], own[n_done: n_done + n_tok + 1]
            e.update(res)
            e["text_equals_plain_decode"] = em == tr
            if em != tr:  # where, and how close the plain decode's two best tokens were there
                i = next((j for j in range(min(len(em), len(tr))) if em[j] != tr[j]), min(len(em), len(tr)))
                e["first_difference"] = {"index": i, "plain_decode_top2_gap": gaps[n_done + i - 1] if n_done + i - 1 < len(gaps) else None}
            n_done += res["tokens"]
        except Exception as ex:  # noqa: BLE001  (a sweep entry must not take the headline down)
            e["error"] = repr(ex)
            out.append(e)
            break
        out.append(e)
    tgt = dr = None
    gc.collect()
    import torch

    torch.cuda.empty_cache()
    return out


def draft_level_entry(args, quick, probe_levels=0, lanes=1):
    """The draft side of cache construction (Cache Construction, eqs. (1)-(9)) as one sweep entry: a
    1B-shaped draft on the whole GPU builds cache levels of K = 100 nodes, top-8 per node, below a
    root behind 1024 tokens of context.  A level is forwarded in ceil(K / 32) calls of the
    draft-mode kernel (tree positions, slots, ancestor mask; per-row top-k and log-sum-exp fused
    into the vocabulary phase), then card_cache_select takes the global top-K of the K * k path
    scores.  Timed: level 2 onwards (parents spread over the level above), host synchronisation
    after every call included.  probe_levels > 0: no timing, that many levels (for counter runs)."""
    import numpy as np
    import torch

    import card_inputs as ci
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape = ci.ModelShape("tiny-draft", 1, 128, 2, 1, 64, 344, 1024) if quick else ci.SHAPES["llama1b"]
    ctx_len, K, k = (64, 40, 4) if quick else (1024, 100, 8)
    n_levels = probe_levels if probe_levels else (2 if quick else 4)
    grid = 0
    if lanes > 1:  # the calls of a level side by side, each on its share of the compute units
        grid = torch.cuda.get_device_properties(0).multi_processor_count // lanes // 8 * 8
    dr = card.Target(shape, ctx_len + 16 + K * (n_levels + 1) + 64, max_r=32, grid_wgs=grid)
    load_synthetic_weights(dr, shape, args.seed + 100)
    if lanes > 1:
        dr.enable_lanes(lanes)
    dev = dr.device
    root = dr.prefill(ci.uniform_tokens(args.seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist())
    mask_base = ctx_len // 16 * 16
    words = (ctx_len + 1 + K * (n_levels + 1) - mask_base + 31) // 32
    assert words <= 32

    def forward(tokens, parents, prev_rows, first, position, sigma):
        """One level: mask rows, the forward calls, the selection of the next level."""
        st, rows = card.card_tree_mask_level(prev_rows, parents, first, ctx_len, mask_base, words)
        assert st == card.CARD_OK
        n = len(tokens)
        tk = torch.empty((n, k), dtype=torch.int32, device=dev)
        tp = torch.empty((n, k), dtype=torch.float32, device=dev)
        calls = 0
        if lanes > 1 and n > 1:
            res = dr.draft_level_wide(ctx_len, tokens, [position] * n, first, rows, mask_base, k)
            tk, tp = res["topk_tokens"], res["topk_probs"]
            calls = (n + 31) // 32
        else:
            for c0 in range(0, n, 32):
                c1 = min(n, c0 + 32)
                res = dr.draft_level(ctx_len, tokens[c0:c1], [position] * (c1 - c0), first + c0, rows[c0:c1], mask_base, k)
                tk[c0:c1], tp[c0:c1] = res["topk_tokens"], res["topk_probs"]
                calls += 1
        ot = torch.empty(K, dtype=torch.int32, device=dev)
        os_ = torch.empty(K, dtype=torch.float32, device=dev)
        op = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = card.card_cache_select(sigma, tk, tp, n, k, K, ot, os_, op, torch.cuda.current_stream(dev).cuda_stream)
        if cnt < 0:
            raise card.CardError(cnt, "card_cache_select")
        torch.cuda.synchronize()
        return rows, ot[:cnt].tolist(), op[:cnt].tolist(), os_[:cnt].clone(), calls

    # level 0: the root alone; its children are level 1
    rows, toks, pars, sigma, _ = forward([root], [-1], None, ctx_len, ctx_len, torch.ones(1, dtype=torch.float32, device=dev))
    first, times, calls = ctx_len + 1, [], 0
    for l in range(1, n_levels + 1):
        t0 = time.perf_counter()
        rows, ntoks, npars, nsigma, c = forward(toks, pars, rows, first, ctx_len + l, sigma)
        if l >= 2 or n_levels == 1:
            times.append((time.perf_counter() - t0) * 1e3)
            calls = c
        first += len(toks)
        n_nodes = len(toks)
        toks, pars, sigma = ntoks, npars, nsigma
    dr = None
    gc.collect()
    torch.cuda.empty_cache()
    if probe_levels:
        return {"draft_probe": True, "levels": n_levels, "K": K, "k": k}
    ms = float(np.median(times))
    params = shape.streamed_weight_bytes() // 2
    rows_issued = 32 * (n_nodes // 32) + (0 if n_nodes % 32 == 0 else (8 if n_nodes % 32 <= 8 else 16 if n_nodes % 32 <= 16 else 32))
    return {"kind": "draft_level", "draft": shape.name, "ctx": ctx_len, "K": n_nodes, "k": k, "calls_per_level": calls,
            "calls_side_by_side": lanes, "workgroups_per_call": grid if grid else "all compute units",
            "ms_per_level": ms, "ms_per_call": ms / calls, "nodes_per_s": n_nodes / (ms * 1e-3),
            "hbm_frac": calls * (shape.streamed_weight_bytes() + shape.kv_bytes(ctx_len)) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            # matrix-pipe work issued: two instructions (high and low activation halves) per weight
            # fragment and 16-row tile, padded rows included, against the dense bf16 peak
            "mfma_tflops_issued": 2 * 2 * rows_issued * params / (ms * 1e-3) / 1e12,
            "mfma_frac_of_bf16_peak": 2 * 2 * rows_issued * params / (ms * 1e-3) / 2.5e15,
            "model_tflops": 2 * n_nodes * params / (ms * 1e-3) / 1e12}


def run_sweep(args, rig8b):
    """Every synthetic configuration besides the headline one.  rig8b: the headline model, reused.
    A section that fails leaves an entry {"section": ..., "error": ...} and the others still run:
    the headline line must not depend on a sweep point."""
    import card_inputs as ci

    out = []
    quick = args.sweep == "quick"
    state = {"decode_tps": None}

    def section(name, fn):
        try:
            fn()
        except Exception as ex:  # noqa: BLE001
            out.append({"section": name, "error": repr(ex)})

    def ctx_sweep():  # context sweep on the 8B shape, r = 8
        for ctx in ([512] if quick else [512, 2048, 8192, 32768]):
            if ctx + 64 > rig8b.tgt.cfg.max_ctx:
                continue
            kind = rig8b.set_context(ctx)
            out.append(sweep_point(rig8b, 8, 10 if quick else 20, kind))

    def decode_8b():  # the target's plain decode rate on the whole GPU (r = 1 steps), the loop's reference
        rig8b.set_context(256 if quick else 1024)
        t0 = time.perf_counter()
        rig8b.greedy(24)
        state["decode_tps"] = 24 / (time.perf_counter() - t0)

    section("llama8b context sweep", ctx_sweep)
    if quick:
        section("llama8b plain decode", decode_8b)
        section("cache loop", lambda: out.append(cache_loop(rig8b, 8, 0.6, 16)))
        section("concurrent loop", lambda: out.extend(concurrent_loop_entries(args, state["decode_tps"], True)))
        section("draft level", lambda: out.append(draft_level_entry(args, True)))
        section("draft level, two calls side by side", lambda: out.append(draft_level_entry(args, True, lanes=2)))
        return out
    rig8b.close()

    def qwen():  # Qwen-7B shape, context 4096: r sweep and the shared-cache loop
        shape = ci.SHAPES["qwen7b"]
        rig = Rig(shape, args.seed, shape.ctx + 160)
        try:
            kind = rig.set_context(shape.ctx)
            for r in (1, 2, 4, 8, 16, 32):
                out.append(sweep_point(rig, r, 20, kind))
            rig.set_context(2048)  # the loop needs the target's real greedy text: a prefilled context
            t0 = time.perf_counter()
            n_dec = 24
            rig.greedy(n_dec)
            decode_tps = n_dec / (time.perf_counter() - t0)
            for p in (0.3, 0.6, 0.9):
                e = cache_loop(rig, 8, p, 96)
                e["plain_decode_tokens_per_s"] = decode_tps
                out.append(e)
        finally:
            rig.close()

    def llama70b():  # 70B shape, context 2048
        shape = ci.SHAPES["llama70b"]
        rig = Rig(shape, args.seed, shape.ctx)
        try:
            kind = rig.set_context(shape.ctx)
            for r in (4, 8, 16):
                out.append(sweep_point(rig, r, 8, kind))
            rig.set_context(1024)
            t0 = time.perf_counter()
            rig.greedy(8)
            state["decode_tps"] = 8 / (time.perf_counter() - t0)  # the 70B target's plain decode rate on the whole GPU
        finally:
            rig.close()

    section("qwen7b r sweep and cache loop", qwen)
    section("llama70b r sweep", llama70b)
    section("concurrent loop", lambda: out.extend(concurrent_loop_entries(args, state["decode_tps"], False)))
    section("draft level", lambda: out.append(draft_level_entry(args, False)))
    section("draft level, two calls side by side", lambda: out.append(draft_level_entry(args, False, lanes=2)))
    return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the verify step on ONE GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import card_inputs as ci
    import paper_2508_04462_amd as card

    shape = ci.SHAPES[args.shape]
    ctx = shape.ctx if args.ctx is None else args.ctx
    r = shape.r if args.r is None else args.r
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.loop_probe:
        print(json.dumps(concurrent_loop_entries(args, None, False)))
        return
    if args.draft_probe:
        print(json.dumps(draft_level_entry(args, False, probe_levels=3)))
        return
    sweep_ctx = 0 if args.sweep == "none" or args.shape != "llama8b" else (512 if args.sweep == "quick" else 32768)
    rig = Rig(shape, args.seed, max(ctx, sweep_ctx))
    rig.set_context(ctx)
    try:
        cands = rig.planted(r)  # planted-prefix invariant on the path being timed
    except RuntimeError as e:
        print(f"bench.py: {e}", file=sys.stderr)
        sys.exit(1)
    cand_dev = torch.tensor(cands, dtype=torch.int32, device=dev)

    if args.timeline is not None:
        print(json.dumps(phase_timeline(rig, ctx, r, cand_dev[r], args.timeline)))
        return
    if args.pmc_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        for i in range(5):
            st = rig.tgt.enqueue_verify(ctx, rig.g0, r, cand=cand_dev[i % (r + 1)])
            assert st == card.CARD_OK
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes": 1 << 30, "verify_steps": 5}))
        return

    ms_per_step, ms_each = rig.time_steps(r, cand_dev, args.steps, args.warmup, min(args.steps, 100))
    kbytes = step_bytes(shape, ctx)
    k_ms = sum(ms_each) / max(len(ms_each), 1)
    achieved = kbytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{args.shape}:ctx{ctx}:r{r}")
            traffic_src = "stored: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under profiles/, not measured in this run"
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
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": kbytes, "avg_launch_us": k_ms * 1e3, "launches_timed": len(ms_each)},
        "paper_context": PAPER_CONTEXT,
    }
    if args.sweep != "none" and args.shape == "llama8b":
        t0 = time.perf_counter()
        out["sweep"] = run_sweep(args, rig)
        out["sweep_seconds"] = time.perf_counter() - t0
    rig.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, args.seed, ctx, r, cands[r])
    card.card_profile_disable()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
