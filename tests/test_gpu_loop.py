"""The query-and-correct loop end to end (overview figure; Cache Correction): a scripted draft
fills the shared candidate cache (host C++ cache of libcard) with a small tree whose best path
follows the target's own greedy text with probability p per token, the target queries the cache
with the token it has just verified, verifies the returned path with card_verify on the GPU,
and corrects the cache with what it accepted.  Whatever the draft's hit rate, the emitted text
must be the target's plain greedy text (lossless at temperature 0), here the CPU oracle's stream
over its decisive prefix; a miss degrades to a plain decode step (r = 1).
"""
import numpy as np
import pytest

import card_inputs as ci
from gpu_common import GAP, make_pair
from oracle import card_oracle as co

pytestmark = pytest.mark.gpu
TINY = ci.SHAPES["tiny"]


def _draft(cache, truth, rng, p, depth, width):
    """Level 0 = the verified token; level i proposes `width` tokens for position i, node 0 the
    best-scored one.  The best path is right with probability p per token; when it goes wrong the
    right token sits on a lower-scored sibling half of the time."""
    cache.write(0, [truth[0]], [-1], [1.0])
    alive = True  # the best path still follows the truth
    for i in range(1, depth):
        if i >= len(truth):
            break
        right = truth[i]
        wrong = [(right + 1 + k) % TINY.vocab for k in range(width)]
        good = alive and rng.random() < p
        toks = [right if good else wrong[0]]
        sibling_right = alive and not good and rng.random() < 0.5
        toks.append(right if sibling_right else wrong[1])
        toks += wrong[2:width]
        scores = [0.9 ** i] + [0.5 ** i * 0.5 ** k for k in range(1, width)]
        cache.write(i, toks, [0] * width, scores)
        alive = good


# seeds whose oracle greedy text stays decisive (top-1 / top-2 gap > 0.05) for 10-20 tokens, found
# by an oracle-only search over seeds 1..42 (about six rows in ten are decisive at this width)
@pytest.mark.parametrize("p,seed", [(0.3, 11), (0.6, 33), (0.9, 42), (1.0, 11), (0.0, 27)])
def test_query_verify_correct_loop_is_lossless(p, seed):
    import paper_2508_04462_amd as card

    shape, n_new, r = TINY, 24, 6
    tgt, w = make_pair(shape, seed, max_ctx=shape.ctx + n_new + r + 16)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    kv_ref = co.OracleKV.empty(shape, shape.ctx + n_new + r + 16)
    g0 = co.prefill(shape, w, kv_ref, ctx)
    want, gaps = co.greedy_decode_cached(shape, w, kv_ref, shape.ctx, g0, n_new)
    decisive_upto = next((i for i, g in enumerate(gaps) if g <= GAP), n_new)
    truth = want[: decisive_upto + 1]  # g0 .. the last token every deciding row of which is decisive
    if len(truth) < 4:
        pytest.skip("seed without a decisive prefix")

    tgt.prefill(ctx)
    cache = card.CandidateCache(K=8, max_depth=r)
    rng = np.random.default_rng(seed)
    n, pending = shape.ctx, g0  # the oracle's pending token starts the stream on both sides
    emitted, hits, misses, accepted = [pending], 0, 0, []
    while len(emitted) < len(truth):
        e = len(emitted) - 1
        _draft(cache, truth[e:] + [0] * r, rng, p, r, 4)
        hit, path, _ = cache.query(pending, r)
        assert hit and path[0] == pending  # the draft has just written the verified token at level 0
        hits += 1
        res = tgt.verify(n, pending, path)
        acc = res["accepted_len"]
        assert 1 <= acc <= len(path)  # the key itself is always accepted
        accepted.append(acc)
        emitted += path[1:acc] + [res["correction_token"]]
        n += res["kv_count"]
        pending = res["correction_token"]
        cache.correct(path[:acc])
        # the sibling branch: if the correction token is still in the tree, the next query hits without a new draft
        hit2, path2, _ = cache.query(pending, r)
        if hit2 and len(emitted) < len(truth):
            assert path2[0] == pending
            res = tgt.verify(n, pending, path2)
            acc = res["accepted_len"]
            assert acc >= 1
            emitted += path2[1:acc] + [res["correction_token"]]
            n += res["kv_count"]
            pending = res["correction_token"]
            cache.correct(path2[:acc])
        else:
            misses += 1
    k = min(len(emitted), len(truth))
    assert emitted[:k] == truth[:k]
    if p == 1.0:
        assert max(accepted) > 1
    if p == 0.0:  # a draft that is always wrong costs nothing but its own work: one token per step
        assert all(a == 1 for a in accepted)


def test_cache_miss_is_a_plain_decode_step():
    import paper_2508_04462_amd as card

    shape, seed = TINY, 7
    tgt, w = make_pair(shape, seed, max_ctx=shape.ctx + 32)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    g0 = tgt.prefill(ctx)
    cache = card.CandidateCache(K=8, max_depth=4)
    hit, path, _ = cache.query(g0, 4)
    assert not hit
    res = tgt.verify(shape.ctx, g0, [g0])  # r = 1: the pending token alone
    assert res["accepted_len"] == 1 and res["kv_count"] == 1
    kv_ref = co.OracleKV.empty(shape, shape.ctx + 32)
    g0_ref = co.prefill(shape, w, kv_ref, ctx)
    if g0_ref == g0:
        ref = co.verify(shape, w, kv_ref, shape.ctx, g0, [g0], keep_logits=True)
        if ref.row_gap[0] > GAP:
            assert res["correction_token"] == ref.correction_token


@pytest.mark.parametrize("flags,p,seed", [(0, 0.6, 33), (0, 0.9, 42), (1, 0.6, 33)], ids=["correct-0.6", "correct-0.9", "query-without-correct"])
def test_step_calls_variable_paths_miss_fallback_and_the_no_correct_variant(flags, p, seed):
    """card_step_begin / card_step_end: one call queries the cache and enqueues the step with
    whatever path length the cache holds (a miss degrades to r = 1 inside the same call), the
    other emits the tokens and corrects the cache - or, with CARD_STEP_NO_CORRECT, leaves it alone
    (the ablation's "query without correct").  The draft writes a fresh tree only every other
    step, paths have ragged lengths, so hits on the sibling branch, hits on a stale tree and
    misses all occur; the text must be the oracle's greedy text whatever happens."""
    import torch

    import paper_2508_04462_amd as card

    shape, n_new, r = TINY, 24, 6
    tgt, w = make_pair(shape, seed, max_ctx=shape.ctx + n_new + r + 16)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    kv_ref = co.OracleKV.empty(shape, shape.ctx + n_new + r + 16)
    g0 = co.prefill(shape, w, kv_ref, ctx)
    want, gaps = co.greedy_decode_cached(shape, w, kv_ref, shape.ctx, g0, n_new)
    decisive_upto = next((i for i, g in enumerate(gaps) if g <= GAP), n_new)
    truth = want[: decisive_upto + 1]
    if len(truth) < 4:
        pytest.skip("seed without a decisive prefix")
    tgt.prefill(ctx)
    cache = card.CandidateCache(K=8, max_depth=r)
    rng = np.random.default_rng(seed)
    staging = torch.zeros(32, dtype=torch.int32).pin_memory()
    out = torch.zeros(4, dtype=torch.int32).pin_memory()
    step = card.CardStep()
    n, pending, emitted = shape.ctx, g0, [g0]
    hits = misses = 0
    lens = set()
    it = 0
    while len(emitted) < len(truth):
        e = len(emitted) - 1
        if it % 2 == 0:  # the draft keeps up only every other step
            depth = 2 + it % (r - 1)  # ragged path lengths
            _draft(cache, truth[e:] + [0] * r, rng, p, depth, 4)
        it += 1
        st = card.card_step_begin(cache.h, tgt.cfg, tgt.packed, tgt.kv(pending), n, r, staging, tgt.workspace,
                                  tgt._stream(), out, tgt.row_argmax, step)
        assert st == card.CARD_OK, card.card_strerror(st)
        torch.cuda.current_stream().synchronize()
        assert 1 <= step.r <= r and step.cand[0] == pending
        hits += step.hit
        misses += 1 - step.hit
        if not step.hit:
            assert step.r == 1
        lens.add(step.r)
        acc, corr, first, count = out.tolist()
        assert 1 <= acc <= step.r and (first, count) == (n, acc)
        st, toks = card.card_step_end(cache.h, step, out, flags)
        assert st == card.CARD_OK and toks == list(step.cand[1:acc]) + [corr]
        emitted += toks
        n += acc
        pending = corr
    k = min(len(emitted), len(truth))
    assert emitted[:k] == truth[:k]
    assert hits >= 1 and len(lens) >= 2
    if flags:  # never corrected: the tree the draft wrote stays as written until the next draft
        assert cache.depth() >= 1


def test_step_calls_at_a_sampling_temperature_emit_the_sampled_text():
    """card_step_begin_sampled: the same loop with the target sampling from the seeded generator
    emits exactly what token-by-token sampling with that seed emits (the text the draft is scripted
    after), with hits, misses and ragged paths on the way."""
    import torch

    import paper_2508_04462_amd as card

    shape, n_new, r, seed, T, sseed = TINY, 24, 6, 8, 1.0, 4242
    tgt, _ = make_pair(shape, seed, max_ctx=shape.ctx + n_new + r + 24)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    tgt.prefill(ctx[:-1])
    g0 = tgt.verify(shape.ctx - 1, -1, [ctx[-1]], temperature=T, seed=sseed)["row_argmax"][0]
    truth, pos = [g0], shape.ctx
    for _ in range(n_new + r):
        truth.append(tgt.verify(pos, truth[-1], [truth[-1]], temperature=T, seed=sseed)["correction_token"])
        pos += 1
    cache = card.CandidateCache(K=8, max_depth=r)
    rng = np.random.default_rng(seed)
    staging = torch.zeros(32, dtype=torch.int32).pin_memory()
    out = torch.zeros(4, dtype=torch.int32).pin_memory()
    step, sampling = card.CardStep(), card.CardSampling(T, sseed)
    n, pending, emitted, hits, it = shape.ctx, g0, [g0], 0, 0
    while len(emitted) < n_new:
        e = len(emitted) - 1
        if it % 2 == 0:
            _draft(cache, truth[e:] + [0] * r, rng, 0.8, 2 + it % (r - 1), 4)
        it += 1
        st = card.card_step_begin_sampled(cache.h, tgt.cfg, tgt.packed, tgt.kv(pending), n, r, staging, tgt.workspace,
                                          tgt._stream(), out, tgt.row_argmax, step, sampling)
        assert st == card.CARD_OK, card.card_strerror(st)
        torch.cuda.current_stream().synchronize()
        hits += step.hit
        acc, corr, first, count = out.tolist()
        assert 1 <= acc <= step.r and (first, count) == (n, acc)
        st, toks = card.card_step_end(cache.h, step, out, 0)
        assert st == card.CARD_OK and toks == list(step.cand[1:acc]) + [corr]
        emitted += toks
        n += acc
        pending = corr
    assert emitted == truth[: len(emitted)]
    assert hits >= 2 and len(emitted) > it  # some steps emitted more than one token
    bad = card.CardSampling(-1.0, 0)
    assert card.card_step_begin_sampled(cache.h, tgt.cfg, tgt.packed, tgt.kv(pending), n, r, staging, tgt.workspace,
                                        tgt._stream(), out, tgt.row_argmax, step, bad) == card.CARD_EINVAL


@pytest.mark.parametrize("p,seed,grids", [(0.7, 11, (128, 64)), (0.95, 42, (192, 64)), (0.0, 27, (64, 32))],
                         ids=["p0.7", "p0.95", "p0"])
def test_concurrent_draft_and_target_on_one_gpu_is_lossless(p, seed, grids):
    """Two models, two host threads, two streams, one GPU: the draft builds cache levels
    (card_draft_level, card_cache_select, card_cache_write) while the target queries, verifies and
    corrects; the kernels share the GPU by compute units.  Whatever the interleaving, the emitted
    text is the target's plain greedy text (checked against the oracle over its decisive prefix
    and against the target's own token-by-token decode beyond it)."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, n_new = TINY, 40
    draft_shape = ci.ModelShape("tiny-draft", 1, 128, 2, 1, 64, 344, 1024, ctx=128, r=4)
    max_ctx = shape.ctx + n_new + 16
    tgt = card.Target(shape, max_ctx, grid_wgs=grids[0])
    load_synthetic_weights(tgt, shape, seed)
    dr = card.Target(draft_shape, shape.ctx + n_new + 16 + 160, grid_wgs=grids[1])
    load_synthetic_weights(dr, draft_shape, seed + 100)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    w = __import__("oracle.from_inputs", fromlist=["oracle_weights"]).oracle_weights(shape, seed)
    kv_ref = co.OracleKV.empty(shape, max_ctx)
    g0_ref = co.prefill(shape, w, kv_ref, ctx)
    want, gaps = co.greedy_decode_cached(shape, w, kv_ref, shape.ctx, g0_ref, n_new)
    decisive_upto = next((i for i, g in enumerate(gaps) if g <= GAP), n_new)
    g0 = tgt.prefill(ctx)
    # the target's own plain decode: what the loop has to reproduce token for token
    own, pos = [g0], shape.ctx
    for _ in range(n_new + 8):
        own.append(tgt.verify(pos, own[-1], [own[-1]])["correction_token"])
        pos += 1
    dr.prefill(ctx)
    # at these sizes the target is the faster model: for the high planted rate it waits for two levels
    # (the draft may run six levels ahead of a target that verifies three tokens per step, so that part of
    # the tree outlives a correction)
    loop = card.ConcurrentLoop(tgt, dr, shape.ctx, g0, K=8, k=4, depth=6 if p >= 0.9 else 3, r_max=3 if p >= 0.9 else None,
                               plant=card.PlantedAgreement(own, p, seed, shape.vocab), wait_levels=2 if p >= 0.9 else 0)
    out = loop.run(n_new)
    assert out["tokens"] >= n_new
    assert loop.emitted[: n_new + 1] == own[: n_new + 1]
    if g0 == g0_ref:
        kk = min(decisive_upto + 1, n_new)
        assert loop.emitted[:kk] == want[:kk]
    assert out["steps"] >= 1 and out["draft_restarts"] >= 1
    if p >= 0.9:
        assert out["mean_accepted_len"] > 1.5 and out["hit_rate"] > 0.5
        # the draft went on below the verified tokens instead of starting a new tree after every step
        assert out["trees_kept_across_corrections"] >= 1
    if p == 0.0:
        assert out["mean_accepted_len"] == 1.0


def test_a_failure_on_the_draft_side_ends_the_loop_with_that_error():
    """Failure handling, forced from the host: the draft thread's planting callback raises after a
    few levels.  run() ends both threads and raises that error (the target does not go on decoding
    against a cache nobody fills); every kernel launched so far finishes normally, and the same
    models run a fresh loop afterwards."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, n_new, seed = TINY, 200, 11
    draft_shape = ci.ModelShape("tiny-draft", 1, 128, 2, 1, 64, 344, 1024, ctx=128, r=4)
    tgt = card.Target(shape, shape.ctx + n_new + 16, grid_wgs=128)
    load_synthetic_weights(tgt, shape, seed)
    dr = card.Target(draft_shape, shape.ctx + n_new + 16 + 160, grid_wgs=64)
    load_synthetic_weights(dr, draft_shape, seed + 100)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    g0 = tgt.prefill(ctx)
    dr.prefill(ctx)
    calls = []

    def failing_plant(index, level, tokens, parents, anchor, parent_tokens):
        calls.append(index)
        if len(calls) == 4:
            raise ValueError("planted failure")
        return list(tokens), list(parents)

    loop = card.ConcurrentLoop(tgt, dr, shape.ctx, g0, K=8, k=4, depth=3, plant=failing_plant)
    with pytest.raises(ValueError, match="planted failure"):
        loop.run(n_new)
    assert len(loop.emitted) - 1 < n_new  # the target stopped early
    # the models are usable afterwards: a fresh loop from the state the first one left
    loop2 = card.ConcurrentLoop(tgt, dr, shape.ctx, g0, K=8, k=4, depth=3)
    tgt.prefill(ctx)
    dr.prefill(ctx)
    out = loop2.run(8)
    assert out["tokens"] >= 8


def test_concurrent_loop_at_temperature_one_emits_the_sampled_text():
    """Temperature 1 in the loop (the paper's T = 1 columns): with the target sampling from the seeded
    generator, the concurrent loop emits exactly what token-by-token sampling with the same seed
    emits, whatever the cache offered."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, n_new, seed, T = TINY, 32, 5, 1.0
    draft_shape = ci.ModelShape("tiny-draft", 1, 128, 2, 1, 64, 344, 1024, ctx=128, r=4)
    tgt = card.Target(shape, shape.ctx + n_new + 24, grid_wgs=128)
    load_synthetic_weights(tgt, shape, seed)
    dr = card.Target(draft_shape, shape.ctx + n_new + 24 + 200, grid_wgs=64)
    load_synthetic_weights(dr, draft_shape, seed + 100)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, shape.ctx, shape.vocab).tolist()
    tgt.prefill(ctx[:-1])
    # the first sampled token: the draw for the position behind the context
    g0 = tgt.verify(shape.ctx - 1, -1, [ctx[-1]], temperature=T, seed=77)["row_argmax"][0]
    own, pos = [g0], shape.ctx
    for _ in range(n_new + 8):
        own.append(tgt.verify(pos, own[-1], [own[-1]], temperature=T, seed=77)["correction_token"])
        pos += 1
    greedy = [g0]
    for i in range(6):
        greedy.append(tgt.verify(shape.ctx + i, greedy[-1], [greedy[-1]])["correction_token"])
    assert greedy != own[:7]  # sampling is not the arg-max here
    dr.prefill(ctx)
    loop = card.ConcurrentLoop(tgt, dr, shape.ctx, g0, K=8, k=4, depth=5, r_max=3, wait_levels=2,
                               plant=card.PlantedAgreement(own, 0.9, seed, shape.vocab), temperature=T, seed=77)
    out = loop.run(n_new)
    assert loop.emitted[: n_new + 1] == own[: n_new + 1]
    assert out["mean_accepted_len"] > 1.3


def test_concurrent_loop_with_a_draft_that_runs_ahead_of_its_target():
    """The paper's regime: the target (8B-shaped, on 192 workgroups) is several times slower than the
    draft (a small model on 64), so the draft builds levels while a verification is in flight, keeps
    its tree across the corrections and the target finds a path below its own token most of the
    time.  The emitted text is the target's plain decode; K = 24 with top-4 per node also takes the
    levels that have fewer extensions than K."""
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    shape, seed, ctx_len, n_new = ci.SHAPES["llama8b"], 3, 256, 96
    draft_shape = ci.ModelShape("small-draft", 2, 512, 8, 2, 64, 1376, shape.vocab, ctx=128, r=4)
    tgt = card.Target(shape, ctx_len + n_new + 64, grid_wgs=192)
    load_synthetic_weights(tgt, shape, seed)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx_len, shape.vocab).tolist()
    g0 = tgt.prefill(ctx)
    own, pos = [g0], ctx_len
    for _ in range(n_new + 16):
        own.append(tgt.verify(pos, own[-1], [own[-1]])["correction_token"])
        pos += 1
    # the second: tree slots run out; the third: the best path is often wrong but a sibling carries the
    # target's token, so the tree is re-rooted on a node that is not the first of its level
    # the fourth: the paper's K = 50 nodes per level (two forward calls per level)
    for K, dmax, p, q in ((8, ctx_len + n_new + 1100, 0.95, 0.0), (24, ctx_len + n_new + 360, 0.95, 0.0),
                          (8, ctx_len + n_new + 1100, 0.5, 0.9), (50, ctx_len + n_new + 1100, 0.95, 0.0)):
        dr = card.Target(draft_shape, dmax, grid_wgs=64)
        load_synthetic_weights(dr, draft_shape, seed + 100)
        dr.prefill(ctx)
        loop = card.ConcurrentLoop(tgt, dr, ctx_len, g0, K=K, k=4, depth=12 if K < 50 else 8, r_max=8,
                                   plant=card.PlantedAgreement(own, p, seed, shape.vocab, q=q))
        out = loop.run(n_new)
        assert loop.emitted[: n_new + 1] == own[: n_new + 1]
        # (thresholds with room for a slower host: the two threads race; measured 2.9-5.6 accepted
        # tokens per step, hit rates 0.72-0.93, 4-6 levels per target step)
        assert out["trees_kept_across_corrections"] > out["draft_restarts"], out
        assert out["draft_levels_per_target_step"] > 1.5, out
        if q == 0.0:
            assert out["mean_accepted_len"] > 1.8 and out["hit_rate"] > 0.45, out
        else:
            # without the siblings every second token would cost a new tree and a plain decode step
            assert out["hit_rate"] > 0.6 and out["draft_restarts"] < 0.5 * out["steps"], out
