"""Host-side driver of the query-and-correct loop with draft and target running concurrently on
ONE GPU (CARD Design, first paragraph: the two models operate in parallel, decoupled by the shared
cache; Experimental Setup: the communication ratio is how many draft levels fit into one target
step).  Nothing is computed here: the draft thread issues card_draft_level / card_cache_select /
card_cache_write, the target thread card_cache_query / card_verify / card_cache_correct, each on
its own HIP stream; the two persistent kernels share the GPU by compute units (cfg.grid_wgs of
the two models add up to at most the number of compute units).

The paper runs the two models on different GPUs; here they share one, so what this loop measures
on top of the paper's scheme is the contention for HBM between the two weight streams.
"""
from __future__ import annotations

import threading
import time
from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding as B
from .runtime import CandidateCache, Target, _lane_streams


def _loop_streams(device):
    """The two streams of the loop: the process-wide pool of side-by-side streams (a process has few
    hardware queues, four by default, and streams are mapped onto them in turn: more streams than
    that end up sharing a queue, and two kernels on one queue run one after the other)."""
    a, b = _lane_streams(device, 2)
    return a, b


class PlantedAgreement:
    """Benchmark / test stand-in for a trained draft (random-init models never agree with each
    other).  For the new level of text position `index`, every node of the level above that carries
    the target's own token of the position before gets, with probability p, the target's token of
    this position as its best-scored child; otherwise, with probability q, as its second-best child
    (a sibling that catches what the best path missed).  The best-scored node of the whole level is
    made a child of the anchor (the best-scored node of the level above that still descends from
    the token verified last), right or wrong by the same draw, so that the best path is the planted
    one; everything else stays as the draft model produced it.  `truth`: the target's own text,
    truth[i] = token of text index i.  Every text index has one draw of each kind, kept for the
    whole run, so a level that is built again says the same thing."""

    def __init__(self, truth: Sequence[int], p: float, seed: int, vocab: int, q: float = 0.0):
        import numpy as np

        self.truth, self.p, self.q, self.vocab = list(truth), p, q, vocab
        self.rng = np.random.default_rng(seed)
        self.draw: Dict[int, tuple] = {}

    def __call__(self, index: int, level: int, tokens: Sequence[int], parents: Sequence[int], anchor: int = 0,
                 parent_tokens: Optional[Sequence[int]] = None):
        tokens, parents = list(tokens), list(parents)
        known = 0 < index < len(self.truth)
        right = self.truth[index] if known else 0
        wrong = (right + 1) % self.vocab
        if index not in self.draw:
            self.draw[index] = (float(self.rng.random()), float(self.rng.random()))
        first, second = self.draw[index][0] < self.p, self.draw[index][1] < self.q

        def on_path(node):
            return known and (parent_tokens is None or parent_tokens[node] == self.truth[index - 1])

        parents[0] = anchor
        tokens[0] = right if on_path(anchor) and first else wrong
        for node in sorted(set(parents)):
            if not on_path(node):
                continue
            kids = [e for e, pa in enumerate(parents) if pa == node]
            if first:
                tokens[kids[0]] = right
            elif second and len(kids) > 1:
                tokens[kids[1]] = right
        return tokens, parents


class _Level:
    """The draft's own record of one cache level: what the cache holds (token, parent, score per
    node) plus where the nodes the draft has forwarded live in its KV cache (slot, mask row) and
    what the forward said about them (top-k tokens and probabilities, device tensors [n][k] with
    token -1 in the rows of nodes that were not forwarded)."""

    def __init__(self, tok, par, score):
        self.tok, self.par, self.score = list(tok), list(par), list(score)
        self.slot: List[Optional[int]] = [None] * len(self.tok)
        self.row: List[Optional[List[int]]] = [None] * len(self.tok)
        self.tk = None
        self.tp = None


def _find(lv: _Level, token: int, parent: int) -> int:
    """The cache's own lookup rule: the best-scored node with this token (below this parent), the
    lowest index among equal scores."""
    best = -1
    for i, t in enumerate(lv.tok):
        if t != token or (parent >= 0 and lv.par[i] != parent):
            continue
        if best < 0 or lv.score[i] > lv.score[best]:
            best = i
    return best


class ConcurrentLoop:
    """target, draft: Target objects on the same device with grid_wgs set so that both kernels fit.
    Both must have the prompt prefilled (context length ctx_len); `pending` is the target's token
    for position ctx_len.  K: nodes per cache level (the paper's 50 or 100 take several forward
    calls per level, 32 rows each), k: top-k per node (K * k <= 2048), depth: levels the
    draft keeps below the token verified last, r_max: tokens the target verifies per step (the
    verified token and at most r_max - 1 levels of the best path; default depth + 1).

    The draft never waits for a verification: it keeps deepening the tree while the target
    verifies, and when the target re-roots the cache (Cache Correction) the draft re-roots its own
    record of the tree the same way and goes on below the surviving subtree; the verified nodes
    stay where they are in the draft's KV cache, visible to their descendants through the mask
    rows those inherited.  Only when the target's own token is not among the candidates (or the
    1024 tree slots behind the draft's dense context are used up) does the draft start a new tree:
    it forwards the tokens committed since the last one as a chain in front of the new root.

    plant(index, level, tokens, parents, anchor, parent_tokens) -> (tokens, parents) lets a benchmark
    overwrite the draft's proposals of one level for text position `index` (random-init models
    never agree, so a planted acceptance rate stands in for the agreement of a trained draft with
    its target); anchor: index, in the level above, of the best-scored node that descends from
    the token verified last; parent_tokens: the tokens of the level above.  None leaves the
    proposals as the draft made them."""

    def __init__(self, target: Target, draft: Target, ctx_len: int, pending: int, K: int = 32, k: int = 8, depth: int = 4,
                 plant: Optional[Callable] = None, wait_levels: int = 0, wait_ms: float = 20.0, r_max: Optional[int] = None,
                 temperature: float = 0.0, seed: int = 0):
        """wait_levels > 0: before a query the target gives the draft up to wait_ms to have that many
        levels in the cache (for set-ups in which the target is the faster model; the paper's target
        is several times slower than its draft and never waits: wait_levels = 0).
        temperature > 0: the target verifies by sampling (one draw per position from the seeded
        counter-based generator): the loop then emits the text of token-by-token sampling with that
        seed, as it emits the greedy text at temperature 0."""
        assert 1 <= K and K * k <= 2048 and 1 <= k <= 16 and depth >= 1  # (the selection pools at most 2048 tuples)
        self.tgt, self.dr = target, draft
        self.K, self.k, self.depth, self.plant = K, k, depth, plant
        self.r_max = min(depth + 1 if r_max is None else r_max, target.cfg.max_r)
        self.wait_levels, self.wait_ms = wait_levels, wait_ms
        self.temperature, self.seed = float(temperature), int(seed)
        self.cache = CandidateCache(K=K, max_depth=depth + 1)
        self.lock = threading.Lock()
        self.t_pos = ctx_len          # target: committed context length
        self.pending = int(pending)   # the token verified last (position t_pos), key of the next query
        self.committed: List[int] = []  # tokens the target has committed behind the prompt
        self.corrections: List[List[int]] = []  # the token lists of the target's corrections, in order
        self.emitted: List[int] = [int(pending)]
        self.d_ctx = ctx_len          # draft: dense context length (prompt + absorbed tokens)
        self.d_absorbed = 0           # committed tokens that are part of the draft's dense context
        self.d_corr_seen = 0
        self.mirror: List[_Level] = []
        self.base_row: Optional[List[int]] = None  # mask row the level-0 nodes inherit (the node verified last)
        self.pos0 = ctx_len           # sequence position of the level-0 nodes
        self.next_slot = ctx_len
        self.mask_base = ctx_len // 16 * 16
        self.words = 1
        self.stop = False
        self.error: Optional[BaseException] = None
        self.stats: Dict[str, float] = {"steps": 0, "hits": 0, "levels": 0, "restarts": 0, "stale_writes": 0,
                                        "rerooted": 0}

    # ---------------------------------------------------------------- target side
    def _target_loop(self, n_tokens: int, stream: torch.cuda.Stream) -> None:
        tgt = self.tgt
        with torch.cuda.stream(stream):
            while len(self.emitted) - 1 < n_tokens and not self.stop:
                if self.wait_levels > 0:
                    t_end = time.perf_counter() + self.wait_ms * 1e-3
                    while self.cache.depth() < self.wait_levels + 1 and time.perf_counter() < t_end and not self.error:
                        time.sleep(0.0001)
                hit, path, _ = self.cache.query(self.pending, self.r_max)
                cand = path if hit else [self.pending]
                res = tgt.verify(self.t_pos, self.pending, cand, temperature=self.temperature, seed=self.seed)
                a = res["accepted_len"]
                if a < 1:
                    raise RuntimeError(f"target step failed: {res}")
                with self.lock:
                    self.cache.correct(cand[:a])
                    self.corrections.append(list(cand[:a]))
                    self.committed += cand[:a]
                    self.t_pos += a
                    self.pending = res["correction_token"]
                    self.emitted += cand[1:a] + [self.pending]
                self.stats["steps"] += 1
                self.stats["hits"] += int(hit)

    # ---------------------------------------------------------------- draft side
    def _mirror_correct(self, toks: Sequence[int]) -> None:
        """card_cache_correct on the draft's record: walk the verified tokens down from level 0,
        keep what hangs strictly below the last one."""
        lv, node = self.mirror, -1
        for d, t in enumerate(toks):
            node = _find(lv[d], t, -1 if d == 0 else node) if d < len(lv) else -1
            if node < 0:
                self.mirror = []
                return
        n = len(toks)
        base_row = lv[n - 1].row[node]
        remap, kept = {node: 0}, []
        for l in range(n, len(lv)):
            src = lv[l]
            keep = [i for i in range(len(src.tok)) if src.par[i] in remap]
            if not keep:
                break
            nl = _Level([src.tok[i] for i in keep], [-1 if l == n else remap[src.par[i]] for i in keep],
                        [src.score[i] for i in keep])
            nl.slot, nl.row = [src.slot[i] for i in keep], [src.row[i] for i in keep]
            if src.tk is not None:
                idx = torch.tensor(keep, dtype=torch.long, device=src.tk.device)
                nl.tk, nl.tp = src.tk.index_select(0, idx), src.tp.index_select(0, idx)
            remap = {old: new for new, old in enumerate(keep)}
            kept.append(nl)
        self.mirror, self.base_row = kept, base_row
        self.pos0 += n
        if kept:
            self.stats["rerooted"] += 1

    def _mirror_matches_cache(self) -> bool:
        if self.cache.depth() != len(self.mirror):
            return False
        for l, lv in enumerate(self.mirror):
            n, tok, par, _ = self.cache.level(l)
            if n != len(lv.tok) or tok != lv.tok or par != lv.par:
                return False
        return True

    def _restart(self, root: int, epoch: int, n_committed: int, root_index: int) -> bool:
        """A new tree below `root`, the target's token at text index root_index.  The draft's dense
        context has to hold everything in front of it: the tokens committed since the last restart
        are forwarded in the same call as the root (a chain in front of it), what does not fit in
        front of that call on its own.  False: the target has moved on meanwhile."""
        dr, k = self.dr, self.k
        new = list(self.committed[self.d_absorbed:n_committed])
        max_r = dr.cfg.max_r
        while len(new) > max_r - 1:
            chunk = new[: max_r - 1]
            dr.verify(self.d_ctx, -1, chunk)
            self.d_ctx += len(chunk)
            self.d_absorbed += len(chunk)
            new = new[len(chunk):]
        ctx_len, n_new = self.d_ctx, len(new)
        root_pos = ctx_len + n_new  # position and slot of the root token
        self.mask_base = ctx_len // 16 * 16
        self.words = min(32, (dr.cfg.max_ctx - self.mask_base + 31) // 32)
        if root_pos + 1 + self.K > min(self.mask_base + 32 * self.words, dr.cfg.max_ctx):
            raise RuntimeError("draft cache too small for the tree")
        if self.cache.write(0, [root], [-1], [1.0], epoch=epoch) != B.CARD_OK:
            self.stats["stale_writes"] += 1
            return False
        self.stats["restarts"] += 1
        # mask rows of the chain [committed tokens ..., root]: each sees the one before it
        chain, prev_row = [], None
        for i in range(n_new + 1):
            st, row = B.card_tree_mask_level(prev_row, [-1 if i == 0 else 0], ctx_len + i, ctx_len, self.mask_base, self.words)
            chain.append(row[0])
            prev_row = row
        res = dr.draft_level(ctx_len, new + [root], [ctx_len + i for i in range(n_new + 1)], ctx_len, chain, self.mask_base, k)
        # the committed tokens are part of the draft's dense context from here on, whatever happens to the tree
        self.d_ctx += n_new
        self.d_absorbed += n_new
        lv = _Level([root], [-1], [1.0])
        lv.slot, lv.row = [root_pos], [chain[-1]]
        lv.tk, lv.tp = res["topk_tokens"][n_new:].clone(), res["topk_probs"][n_new:].clone()
        self.mirror, self.base_row, self.pos0, self.next_slot = [lv], None, root_pos, root_pos + 1
        return True

    def _forward(self, D: int, alive: Sequence[int]) -> None:
        """Forward the nodes `alive` of level D: their keys and values go to fresh slots, their top-k
        into the level's record."""
        dr, lv, dev = self.dr, self.mirror[D], self.dr.device
        first = self.next_slot
        if D == 0:
            st, rows = B.card_tree_mask_level(None if self.base_row is None else [self.base_row],
                                              [-1 if self.base_row is None else 0] * len(alive), first, self.d_ctx,
                                              self.mask_base, self.words)
        else:
            up = self.mirror[D - 1]
            st, rows = B.card_tree_mask_level([up.row[lv.par[i]] for i in alive], list(range(len(alive))), first, self.d_ctx,
                                              self.mask_base, self.words)
        if st != B.CARD_OK:
            raise B.CardError(st, "card_tree_mask_level")
        n = len(lv.tok)
        lv.tk = torch.full((n, self.k), -1, dtype=torch.int32, device=dev)
        lv.tp = torch.zeros((n, self.k), dtype=torch.float32, device=dev)
        toks = [lv.tok[i] for i in alive]
        for c0 in range(0, len(alive), 32):  # a level wider than one call: peers never see each other
            c1 = min(len(alive), c0 + 32)
            res = dr.draft_level(self.d_ctx, toks[c0:c1], [self.pos0 + D] * (c1 - c0), first + c0, rows[c0:c1], self.mask_base,
                                 self.k)
            idx = torch.tensor(list(alive[c0:c1]), dtype=torch.long, device=dev)
            lv.tk.index_copy_(0, idx, res["topk_tokens"])
            lv.tp.index_copy_(0, idx, res["topk_probs"])
        for j, i in enumerate(alive):
            lv.slot[i], lv.row[i] = first + j, rows[j]
        self.next_slot += len(alive)

    def _draft_loop(self, stream: torch.cuda.Stream) -> None:
        K, k, dev = self.K, self.k, self.dr.device
        with torch.cuda.stream(stream):
            while not self.stop:
                with self.lock:
                    fresh = self.corrections[self.d_corr_seen:]
                    self.d_corr_seen = len(self.corrections)
                    for toks in fresh:
                        if self.mirror:
                            self._mirror_correct(toks)
                    epoch, root, n_committed = self.cache.epoch(), self.pending, len(self.committed)
                    root_index = len(self.emitted) - 1  # text index of the token verified last
                    if fresh and self.mirror and not self._mirror_matches_cache():
                        raise RuntimeError("the draft's record of the tree and the cache disagree")
                i0 = _find(self.mirror[0], root, -1) if self.mirror else -1
                limit = min(self.mask_base + 32 * self.words, self.dr.cfg.max_ctx)
                if i0 < 0 or self.next_slot + K > limit:
                    self._restart(root, epoch, n_committed, root_index)
                    continue
                # nodes below the verified token, level by level; the tree grows below the deepest of them
                alive = [[i0]]
                for l in range(1, len(self.mirror)):
                    up = set(alive[-1])
                    cur = [i for i, p in enumerate(self.mirror[l].par) if p in up]
                    if not cur:
                        break
                    alive.append(cur)
                D = len(alive) - 1
                if D >= self.depth:
                    # the tree is as deep as it gets: wait for the target's next correction
                    while not self.stop and self.cache.epoch() == epoch:
                        time.sleep(0.0002)
                    continue
                lv = self.mirror[D]
                todo = [i for i in alive[D] if lv.slot[i] is None]
                if lv.tk is None:
                    self._forward(D, alive[D])
                elif todo:
                    raise RuntimeError("a node below the verified token was never forwarded")
                tk = lv.tk
                if len(alive[D]) < len(lv.tok):
                    dead = torch.tensor([i for i in range(len(lv.tok)) if i not in set(alive[D])], dtype=torch.long, device=dev)
                    tk = lv.tk.clone()
                    tk.index_fill_(0, dead, -1)
                sigma = torch.tensor(lv.score, dtype=torch.float32, device=dev)
                ot = torch.empty(K, dtype=torch.int32, device=dev)
                os_ = torch.empty(K, dtype=torch.float32, device=dev)
                op = torch.empty(K, dtype=torch.int32, device=dev)
                cnt = B.card_cache_select(sigma, tk, lv.tp, len(lv.tok), k, K, ot, os_, op, stream.cuda_stream)
                if cnt < 0:
                    raise B.CardError(cnt, "card_cache_select")
                stream.synchronize()
                nt, npar, ns = ot[:cnt].tolist(), op[:cnt].tolist(), os_[:cnt].tolist()
                if -1 in nt:  # fewer tuples than K below the nodes that are left: the rest is marked empty
                    cnt = nt.index(-1)
                    nt, npar, ns = nt[:cnt], npar[:cnt], ns[:cnt]
                if cnt == 0:
                    raise RuntimeError("no extension below the verified token")
                if self.plant is not None:
                    anchor = alive[D][0]  # the best-scored node of this level below the verified token
                    nt, npar = self.plant(root_index + D + 1, D + 1, nt, npar, anchor, lv.tok)
                if self.stop or self.cache.write(D + 1, nt, npar, ns, epoch=epoch) != B.CARD_OK:
                    self.stats["stale_writes"] += 1
                    continue  # the target has corrected the cache meanwhile: what was forwarded stays on record
                self.stats["levels"] += 1
                self.mirror = self.mirror[: D + 1] + [_Level(nt, npar, ns)]

    # ---------------------------------------------------------------- run
    def run(self, n_tokens: int) -> Dict[str, float]:
        s_t, s_d = _loop_streams(self.tgt.device)

        def guard(fn, *args):
            try:
                fn(*args)
            except BaseException as e:  # noqa: BLE001  (reported by run(); the first one wins, and ends both threads)
                if self.error is None:
                    self.error = e
                self.stop = True
            finally:
                if fn == self._target_loop:
                    self.stop = True

        td = threading.Thread(target=guard, args=(self._draft_loop, s_d))
        tt = threading.Thread(target=guard, args=(self._target_loop, n_tokens, s_t))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        td.start()
        tt.start()
        tt.join()
        dt = time.perf_counter() - t0
        self.stop = True
        td.join()
        if self.error is not None:
            raise self.error
        n = len(self.emitted) - 1
        steps = max(self.stats["steps"], 1)
        return {"tokens": n, "seconds": dt, "accepted_tokens_per_s": n / dt, "steps": self.stats["steps"],
                "mean_accepted_len": n / steps, "hit_rate": self.stats["hits"] / steps,
                "draft_levels_per_target_step": self.stats["levels"] / steps, "draft_restarts": self.stats["restarts"],
                "stale_writes": self.stats["stale_writes"], "trees_kept_across_corrections": self.stats["rerooted"],
                "ms_per_target_step": dt * 1e3 / steps}
