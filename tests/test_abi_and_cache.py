"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, sizes and
argument errors come from host code, and the host-side candidate cache agrees with its oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import card_inputs as ci
import paper_2508_04462_amd as card
from oracle.cache_oracle import CandidateCacheOracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "card.h")).read()
    names = set(re.findall(r"\b(card_[a-z_]+)\s*\(", header))
    assert {"card_verify", "card_cache_query", "card_cache_write", "card_cache_correct"} <= names
    for n in sorted(names):
        assert hasattr(card.lib, n), n


def test_sizes_follow_the_shapes():
    shape = ci.SHAPES["llama8b"]
    cfg = card.make_cfg(shape, 2048)
    wb = card.card_packed_weight_bytes(cfg)
    # streamed bf16 weights + the embedding table + gains, a little tile padding
    expect = shape.streamed_weight_bytes() + 2 * shape.vocab * shape.d_model
    assert expect <= wb <= expect * 1.001
    assert card.card_kv_pool_bytes(cfg, 128) == 32 * 128 * 8 * 16 * 128 * 2
    assert card.card_workspace_bytes(cfg) > 32 * 4096 * 4
    bad = card.make_cfg(shape, 2048)
    bad.head_dim = 96
    assert card.card_packed_weight_bytes(bad) == 0 and card.card_workspace_bytes(bad) == 0


@pytest.mark.parametrize("n_tiles,k_steps,batch,grid", [(384, 128, 2, 256), (256, 448, 1, 256), (1792, 128, 8, 256),
                                                        (8016, 128, 8, 256), (43, 9, 2, 7), (5, 3, 8, 16), (64, 8, 1, 256)])
def test_stream_order_is_a_bijection_with_contiguous_runs(n_tiles, k_steps, batch, grid):
    """The packed order of a matrix: every fragment exactly once, and the fragments of one
    (grid position, wavefront pair) form ONE run ordered batch, then k-step, then tile."""
    idx = np.array([[card.card_stream_frag_index(n_tiles, k_steps, batch, grid, t, s) for s in range(k_steps)]
                    for t in range(n_tiles)], dtype=np.int64)
    assert sorted(idx.ravel().tolist()) == list(range(n_tiles * k_steps))
    nxt = 0
    for p in range(grid):
        tiles = list(range(p, n_tiles, grid))
        for w in range(4):
            s0, s1 = w * k_steps // 4, (w + 1) * k_steps // 4
            for b in range(0, len(tiles), batch):
                for s in range(s0, s1):
                    for t in tiles[b:b + batch]:
                        assert idx[t, s] == nxt, (p, w, b, s, t)
                        nxt += 1
    assert nxt == n_tiles * k_steps
    assert card.card_stream_frag_index(n_tiles, k_steps, batch, grid, n_tiles, 0) == -1
    assert card.card_stream_frag_index(n_tiles, k_steps, batch, 0, 0, 0) == -1


def test_argument_errors_are_caught_on_the_host():
    cfg = card.make_cfg(ci.SHAPES["tiny"], 256)
    kv = card.CardKV(0x1000, 0x1000, 0x1000, 16, -1)
    assert card.card_verify(cfg, None, kv, 0, 0x1000, 1, 0x1000, None, 0x1000) == card.CARD_EINVAL
    assert card.card_verify(cfg, 0x1000, kv, 0, 0x1000, 0, 0x1000, None, 0x1000) == card.CARD_ERANGE
    assert card.card_verify(cfg, 0x1000, kv, 0, 0x1000, 33, 0x1000, None, 0x1000) == card.CARD_ERANGE
    assert card.card_verify(cfg, 0x1000, kv, 250, 0x1000, 8, 0x1000, None, 0x1000) == card.CARD_ECAPACITY
    assert card.card_verify(cfg, 0x1000, kv, -1, 0x1000, 8, 0x1000, None, 0x1000) == card.CARD_EINVAL
    assert card.card_weights_pack_tensor(cfg, 99, 0, 0x1000, 0x1000) == card.CARD_EINVAL
    assert card.card_weights_pack_tensor(cfg, card.TENSOR_IDS["wq"], 7, 0x1000, 0x1000) == card.CARD_ERANGE
    assert card.card_strerror(card.CARD_ECAPACITY) == "KV cache capacity exceeded"


# ------------------------------------------------------------------------------- candidate cache


def _random_tree(rng, K, depth, vocab):
    levels = []
    prev = 0
    for l in range(depth):
        n = int(rng.integers(1, K + 1))
        toks = rng.integers(0, vocab, size=n).tolist()
        parents = [-1] * n if l == 0 else rng.integers(0, prev, size=n).tolist()
        scores = (rng.integers(1, 64, size=n) / 64.0).tolist()  # exact in fp32, ties happen
        levels.append((toks, parents, scores))
        prev = n
    return levels


def _same(lib_cache, ora):
    assert lib_cache.depth() == ora.depth()
    for l, lv in enumerate(ora.levels):
        n, t, p, s = lib_cache.level(l)
        assert (n, t, p) == (len(lv.tokens), lv.tokens, lv.parents)
        np.testing.assert_allclose(s, lv.scores)


@pytest.mark.parametrize("seed", range(12))
def test_cache_matches_oracle_on_random_trees(seed):
    rng = np.random.default_rng(seed)
    K, depth, vocab = 6, 5, 7  # a tiny vocabulary forces duplicate tokens
    c = card.CandidateCache(K, depth)
    o = CandidateCacheOracle(K, depth)
    for _ in range(6):
        for l, (t, p, s) in enumerate(_random_tree(rng, K, depth, vocab)):
            assert c.write(l, t, p, s) == card.CARD_OK
            o.write_level(l, t, p, s)
        _same(c, o)
        for tok in range(vocab):
            for max_len in (1, 2, 3, 9):
                hit, path, score = c.query(tok, max_len)
                ohit, opath, oscore = o.query(tok, max_len)
                assert (hit, path) == (ohit, opath)
                assert abs(score - oscore) < 1e-6
        # walk a verified chain that mostly follows the tree and sometimes leaves it
        chain = []
        node_tok = o.levels[0].tokens[int(rng.integers(len(o.levels[0].tokens)))]
        hit, path, _ = o.query(node_tok, int(rng.integers(1, depth + 1)))
        chain = list(path)
        if rng.random() < 0.3:
            chain.append(vocab + 1)
        assert c.correct(chain) == o.correct(chain)
        _same(c, o)
        assert c.epoch() == o.epoch
        # refill below what is left, as the draft side would
        base = o.depth()
        for l in range(base, depth):
            n_prev = len(o.levels[l - 1].tokens) if l else 0
            n = int(rng.integers(1, K + 1))
            t = rng.integers(0, vocab, size=n).tolist()
            p = [-1] * n if l == 0 else rng.integers(0, n_prev, size=n).tolist()
            s = (rng.integers(1, 64, size=n) / 64.0).tolist()
            assert c.write(l, t, p, s) == card.CARD_OK
            o.write_level(l, t, p, s)
        _same(c, o)


def test_cache_write_errors_and_stale_epoch():
    c = card.CandidateCache(4, 3)
    assert c.write(1, [1], [0], [0.5]) == card.CARD_ERANGE  # level 0 missing
    assert c.write(0, [1, 2], [-1, -1], [0.6, 0.4]) == card.CARD_OK
    assert c.write(0, [1, 2], [0, -1], [0.6, 0.4]) == card.CARD_ERANGE  # level-0 parents must be -1
    assert c.write(1, [3], [2], [0.5]) == card.CARD_ERANGE  # parent outside level 0
    assert c.write(1, [1, 2, 3, 4, 5], [0] * 5, [0.1] * 5) == card.CARD_ERANGE  # more than K nodes
    assert c.write(1, [3], [1], [0.5]) == card.CARD_OK
    assert c.write(3, [3], [0], [0.5]) == card.CARD_ERANGE  # beyond max_depth
    e = c.epoch()
    assert c.correct([2])
    assert c.write(1, [9], [0], [0.5], epoch=e) == card.CARD_ESTALE  # the writer missed a correction
    assert c.level(0)[1] == [3]
    assert c.write(1, [9], [0], [0.5]) == card.CARD_OK


def test_cache_concurrent_writer_and_reader_do_not_corrupt():
    import threading

    c = card.CandidateCache(8, 4)
    stop = threading.Event()
    errors = []

    def writer():
        rng = np.random.default_rng(0)
        while not stop.is_set():
            ep = c.epoch()
            prev = 0
            for l in range(4):
                n = int(rng.integers(1, 9))
                p = [-1] * n if l == 0 else rng.integers(0, prev, size=n).tolist()
                st = c.write(l, rng.integers(0, 5, size=n).tolist(), p, rng.random(n).tolist(), epoch=ep)
                if st == card.CARD_ESTALE:
                    break
                if st != card.CARD_OK:
                    errors.append(st)
                prev = n

    th = threading.Thread(target=writer)
    th.start()
    try:
        for i in range(3000):
            hit, path, _ = c.query(i % 5, 4)
            assert len(path) <= 4 and (not hit or path[0] == i % 5)
            if i % 7 == 0:
                c.correct(path[:2])
    finally:
        stop.set()
        th.join()
    assert not errors


def test_step_end_emits_and_corrects_on_the_host():
    """card_step_end is host logic: accepted path tokens behind the query key, then the target's own
    token; the cache is re-rooted at the accepted candidates unless the no-correct flag is set."""
    import ctypes as C

    def tree():
        c = card.CandidateCache(K=4, max_depth=4)
        c.write(0, [10], [-1], [1.0])
        c.write(1, [11, 21], [0, 0], [0.9, 0.4])
        c.write(2, [12, 22, 32], [0, 0, 1], [0.8, 0.3, 0.2])
        return c

    step = card.CardStep()
    step.r, step.hit = 3, 1
    step.cand[0], step.cand[1], step.cand[2] = 10, 11, 12
    out = (C.c_int32 * 4)(2, 22, 100, 2)  # accepted the key and 11, the target's own next token is 22
    c = tree()
    st, toks = card.card_step_end(c.h, step, C.addressof(out), 0)
    assert st == card.CARD_OK and toks == [11, 22]
    n, t, p, s = c.level(0)  # level 0 now holds the children of node 11
    assert sorted(t) == [12, 22]
    hit, path, _ = c.query(22, 4)
    assert hit and path == [22]
    c2 = tree()
    st, toks = card.card_step_end(c2.h, step, C.addressof(out), card.CARD_STEP_NO_CORRECT)
    assert st == card.CARD_OK and toks == [11, 22]
    assert c2.level(0)[1] == [10] and c2.depth() == 3  # untouched
    bad = (C.c_int32 * 4)(-1, -1, 100, 0)  # a failed step must not touch the cache
    st, toks = card.card_step_end(c2.h, step, C.addressof(bad), 0)
    assert st == card.CARD_EDEVICE and c2.level(0)[1] == [10]
    over = (C.c_int32 * 4)(4, 5, 100, 4)  # more accepted than forwarded
    assert card.card_step_end(c2.h, step, C.addressof(over), 0)[0] == card.CARD_EDEVICE


def test_step_begin_argument_errors():
    cfg = card.make_cfg(ci.SHAPES["tiny"], 256, max_r=8)
    c = card.CandidateCache(K=4, max_depth=4)
    step = card.CardStep()
    kv = card.CardKV(0x1000, 0x1000, 0x1000, 16, 5)
    assert card.card_step_begin(c.h, cfg, 0x1000, kv, 0, 0, 0x1000, 0x1000, None, 0x1000, None, step) == card.CARD_ERANGE
    assert card.card_step_begin(c.h, cfg, 0x1000, kv, 0, 9, 0x1000, 0x1000, None, 0x1000, None, step) == card.CARD_ERANGE
    no_pending = card.CardKV(0x1000, 0x1000, 0x1000, 16, -1)
    assert card.card_step_begin(c.h, cfg, 0x1000, no_pending, 0, 4, 0x1000, 0x1000, None, 0x1000, None, step) == card.CARD_EINVAL
    assert card.card_step_begin(None, cfg, 0x1000, kv, 0, 4, 0x1000, 0x1000, None, 0x1000, None, step) == card.CARD_EINVAL
    smp = card.CardSampling(1.0, 7)
    assert card.card_step_begin_sampled(c.h, cfg, 0x1000, kv, 0, 0, 0x1000, 0x1000, None, 0x1000, None, step, smp) == card.CARD_ERANGE
    assert card.card_step_begin_sampled(c.h, cfg, 0x1000, kv, 0, 4, 0x1000, 0x1000, None, 0x1000, None, step,
                                        card.CardSampling(-2.0, 7)) == card.CARD_EINVAL


def test_tree_mask_level_matches_the_mask_oracle():
    """Host mask builder against oracle/cache_oracle.tree_mask (ancestor inheritance + identity,
    peers invisible) on random trees, with the context bits below the first tree slot."""
    from oracle.cache_oracle import tree_mask

    rng = np.random.default_rng(3)
    for ctx_len, widths in [(37, [3, 5, 4, 6]), (16, [1, 2, 9]), (95, [7, 7, 7, 7, 7])]:
        parents = [[-1] * widths[0]] + [rng.integers(0, widths[l - 1], size=widths[l]).tolist() for l in range(1, len(widths))]
        ref = tree_mask(parents)
        offs = np.cumsum([0] + widths)
        mask_base = ctx_len // 16 * 16
        tree_base = (ctx_len + 15) // 16 * 16
        words = (tree_base + int(offs[-1]) - mask_base + 31) // 32
        prev = None
        for l, par in enumerate(parents):
            st, rows = card.card_tree_mask_level(prev, par, tree_base + int(offs[l]), ctx_len, mask_base, words)
            assert st == card.CARD_OK
            for i, row in enumerate(rows):
                bits = {mask_base + 32 * w + b for w in range(words) for b in range(32) if (row[w] >> b) & 1}
                want = set(range(mask_base, ctx_len)) | {tree_base + int(j) for j in np.flatnonzero(ref[offs[l] + i])}
                assert bits == want, (l, i)
            prev = rows
    assert card.card_tree_mask_level(None, [0], 48, 37, 32, 2)[0] == card.CARD_EINVAL  # a parent without rows
    assert card.card_tree_mask_level(None, [-1], 30, 37, 32, 2)[0] == card.CARD_ERANGE  # slot inside the context
    assert card.card_tree_mask_level(None, [-1], 48, 37, 40, 2)[0] == card.CARD_EINVAL  # base not on a page boundary


@pytest.mark.parametrize("seed", range(8))
def test_the_draft_loop_rerooting_of_its_own_tree_record_follows_the_cache(seed):
    """The concurrent loop's draft keeps a record of the tree beside the cache (slots and mask rows
    of the nodes it has forwarded) and re-roots it itself after every correction: same lookup rule,
    same surviving nodes in the same order, same parent indices as card_cache_correct."""
    from paper_2508_04462_amd.loop import ConcurrentLoop, _Level

    rng = np.random.default_rng(100 + seed)
    K, depth, vocab = 6, 5, 5
    loop = object.__new__(ConcurrentLoop)
    loop.cache = card.CandidateCache(K, depth)
    loop.mirror, loop.base_row, loop.pos0 = [], None, 40
    loop.stats = {"rerooted": 0}
    for _ in range(8):
        # (re)fill below what is left, as the draft would; forwarded nodes get a slot and a row tag
        for l in range(len(loop.mirror), depth):
            n_prev = len(loop.mirror[l - 1].tok) if l else 0
            n = int(rng.integers(1, K + 1))
            t = rng.integers(0, vocab, size=n).tolist()
            p = [-1] * n if l == 0 else rng.integers(0, n_prev, size=n).tolist()
            s = (rng.integers(1, 64, size=n) / 64.0).tolist()
            assert loop.cache.write(l, t, p, s) == card.CARD_OK
            lv = _Level(t, p, s)
            lv.slot = [1000 * l + i for i in range(n)]
            lv.row = [[l, i] for i in range(n)]
            loop.mirror.append(lv)
        assert loop._mirror_matches_cache()
        tok0 = loop.mirror[0].tok[int(rng.integers(len(loop.mirror[0].tok)))]
        hit, chain, _ = loop.cache.query(tok0, int(rng.integers(1, depth + 1)))
        assert hit
        if rng.random() < 0.25:
            chain = chain + [vocab + 3]  # leaves the tree: both sides end up empty
        pos_before, last = loop.pos0, None
        # the record's row of the node verified last is what the new level 0 inherits
        node = -1
        for d, t in enumerate(chain):
            if d >= len(loop.mirror):
                node = -1
                break
            cands = [i for i, tt in enumerate(loop.mirror[d].tok) if tt == t and (d == 0 or loop.mirror[d].par[i] == node)]
            if not cands:
                node = -1
                break
            node = max(cands, key=lambda i: (loop.mirror[d].score[i], -i))
            last = loop.mirror[d].row[node]
        loop.cache.correct(chain)
        loop._mirror_correct(chain)
        assert loop._mirror_matches_cache()
        if loop.mirror:
            assert node >= 0 and loop.base_row == last and loop.pos0 == pos_before + len(chain)
            # slots and rows travelled with their nodes
            for lv in loop.mirror:
                assert all(r[1] == s % 1000 for r, s in zip(lv.row, lv.slot))


def test_argument_errors_of_the_later_entry_points_are_caught_on_the_host():
    """Sampled, static, draft-level and selection calls refuse bad arguments before anything is
    enqueued (fake device addresses: nothing here may reach a launch)."""
    cfg = card.make_cfg(ci.SHAPES["tiny"], 256)
    kv = card.CardKV(0x1000, 0x1000, 0x1000, 16, -1)
    P = 0x1000
    # sampling: the temperature must be a number >= 0
    assert card.card_verify_sampled(cfg, P, kv, 0, P, 4, card.CardSampling(-1.0, 0), P, None, P) == card.CARD_EINVAL
    assert card.card_verify_sampled(cfg, P, kv, 0, P, 4, card.CardSampling(float("nan"), 0), P, None, P) == card.CARD_EINVAL
    assert card.card_verify_sampled(cfg, P, kv, 0, P, 40, card.CardSampling(1.0, 0), P, None, P) == card.CARD_ERANGE
    # the entry point without allocation refuses a model whose workspace exceeds its scratch array
    big = card.make_cfg(ci.SHAPES["llama70b"], 4096)
    assert card.card_workspace_bytes(big) > card.card_static_scratch_bytes()
    assert card.card_verify_static(big, P, kv, 0, P, 4, None, P) == card.CARD_ETOOBIG
    assert card.card_verify_static(cfg, None, kv, 0, P, 4, None, P) == card.CARD_EINVAL
    assert card.card_verify_static(cfg, P, kv, 0, P, 0, None, P) == card.CARD_ERANGE
    # draft level: k, mask geometry, slots
    def rows(first, words, base):
        return card.CardTreeRows(P, P, first, P, words, base)
    tk = P
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 2, 64), 4, 0, P, None, tk, P) == card.CARD_ERANGE      # k = 0
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 2, 64), 4, 17, P, None, tk, P) == card.CARD_ERANGE     # k > 16
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 33, 64), 4, 4, P, None, tk, P) == card.CARD_ERANGE     # 33 mask words
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 2, 60), 4, 4, P, None, tk, P) == card.CARD_EINVAL      # base off a page
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 2, 80), 4, 4, P, None, tk, P) == card.CARD_EINVAL      # base behind the context
    assert card.card_draft_level(cfg, P, kv, 64, rows(60, 2, 48), 4, 4, P, None, tk, P) == card.CARD_ERANGE      # slot inside the context
    assert card.card_draft_level(cfg, P, kv, 64, rows(126, 2, 64), 4, 4, P, None, tk, P) == card.CARD_ERANGE     # rows past the mask
    assert card.card_draft_level(cfg, P, kv, 64, rows(254, 8, 64), 4, 4, P, None, tk, P) == card.CARD_ECAPACITY  # past max_ctx
    assert card.card_draft_level(cfg, P, kv, 64, rows(64, 2, 64), 4, 4, P, None, None, P) == card.CARD_EINVAL
    # selection
    assert card.card_cache_select(P, P, P, 0, 4, 8, P, P, P) == card.CARD_ERANGE
    assert card.card_cache_select(P, P, P, 200, 16, 8, P, P, P) == card.CARD_ERANGE  # more than 2048 tuples
    assert card.card_cache_select(P, None, P, 4, 4, 8, P, P, P) == card.CARD_EINVAL


def test_planted_agreement_is_per_text_index_and_follows_every_on_path_parent():
    """The benchmark's stand-in for a trained draft: one draw per text index (a level that is built
    twice says the same thing), the target's token below every node that carries the target's
    previous token, the best node of the level below the anchor, a sibling where the best misses."""
    from paper_2508_04462_amd.loop import PlantedAgreement

    truth = list(range(100, 140))
    always = PlantedAgreement(truth, 1.0, 1, 1000)
    toks, pars = always(5, 2, [7, 8, 9, 10], [1, 1, 2, 2], anchor=2, parent_tokens=[0, truth[4], truth[4]])
    assert pars[0] == 2 and toks[0] == truth[5]          # best node: below the anchor, right
    assert toks[1] == truth[5] and pars[1] == 1          # the other on-path parent gets its right child too
    never = PlantedAgreement(truth, 0.0, 1, 1000)
    toks, pars = never(5, 2, [7, 8, 9, 10], [1, 1, 2, 2], anchor=2, parent_tokens=[0, truth[4], truth[4]])
    assert truth[5] not in toks and pars[0] == 2
    sib = PlantedAgreement(truth, 0.0, 1, 1000, q=1.0)
    toks, pars = sib(5, 2, [7, 8, 9, 10], [2, 2, 1, 1], anchor=2, parent_tokens=[0, truth[4], truth[4]])
    assert toks[0] != truth[5] and toks[1] == truth[5] and toks[3] == truth[5] and toks[2] != truth[5]
    # an anchor that is off the target's text gets nothing right
    toks, _ = always(5, 2, [7, 8], [0, 0], anchor=0, parent_tokens=[55])
    assert truth[5] not in toks
    # the same index twice: the same decision
    half = PlantedAgreement(truth, 0.5, 3, 1000)
    first = [half(i, 1, [1, 2], [0, 0], 0, [truth[i - 1]])[0] for i in range(1, 30)]
    again = [half(i, 1, [1, 2], [0, 0], 0, [truth[i - 1]])[0] for i in range(1, 30)]
    assert first == again and 5 < sum(t[0] == truth[i] for i, t in zip(range(1, 30), first)) < 25
