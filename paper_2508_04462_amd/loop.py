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
from .runtime import CandidateCache, Target


_STREAMS: Dict[str, tuple] = {}


def _loop_streams(device):
    """One pair of streams per device for the life of the process.  A process has few hardware queues
    (four by default) and streams are mapped onto them in turn: fresh streams for every loop end up
    sharing a queue sooner or later, and the two kernels then run one after the other, not side by
    side."""
    key = str(device)
    if key not in _STREAMS:
        _STREAMS[key] = (torch.cuda.Stream(device=device), torch.cuda.Stream(device=device))
    return _STREAMS[key]


class PlantedAgreement:
    """Benchmark / test stand-in for a trained draft (random-init models never agree with each
    other): per text position the best-scored node of a level is made to carry the target's own
    token with probability p as long as the best path has been right so far, and to hang below the
    best node of the level above; everything else stays as the draft model produced it.  `truth`:
    the target's own text, truth[i] = token of text index i."""

    def __init__(self, truth: Sequence[int], p: float, seed: int, vocab: int):
        import numpy as np

        self.truth, self.p, self.vocab = list(truth), p, vocab
        self.rng = np.random.default_rng(seed)
        self.alive = True

    def __call__(self, index: int, level: int, tokens: Sequence[int], parents: Sequence[int]):
        if level == 1:
            self.alive = True
        tokens, parents = list(tokens), list(parents)
        known = index < len(self.truth)
        right = self.truth[index] if known else 0
        good = self.alive and known and self.rng.random() < self.p
        tokens[0] = right if good else (right + 1) % self.vocab
        parents[0] = 0
        self.alive = good
        return tokens, parents


class ConcurrentLoop:
    """target, draft: Target objects on the same device with grid_wgs set so that both kernels fit.
    Both must have the prompt prefilled (context length ctx_len); `pending` is the target's token
    for position ctx_len.  K (<= 32): nodes per cache level, k: top-k per node, depth: levels the
    draft builds below the verified token (a path carries at most depth + 1 tokens).

    plant(index, level, tokens, parents) -> (tokens, parents) lets a benchmark overwrite the draft's
    proposals of one level for text position `index` (random-init models never agree, so a planted
    acceptance rate stands in for the agreement of a trained draft with its target); None leaves
    them as the draft made them."""

    def __init__(self, target: Target, draft: Target, ctx_len: int, pending: int, K: int = 32, k: int = 8, depth: int = 4,
                 plant: Optional[Callable] = None, wait_levels: int = 0, wait_ms: float = 20.0):
        """wait_levels > 0: before a query the target gives the draft up to wait_ms to have that many
        levels in the cache (for set-ups in which the target is the faster model; the paper's target
        is several times slower than its draft and never waits: wait_levels = 0)."""
        assert 1 <= K <= 32 and 1 <= k <= 16 and depth >= 1
        self.tgt, self.dr = target, draft
        self.K, self.k, self.depth, self.plant = K, k, depth, plant
        self.wait_levels, self.wait_ms = wait_levels, wait_ms
        self.cache = CandidateCache(K=K, max_depth=depth + 1)
        self.lock = threading.Lock()
        self.t_pos = ctx_len          # target: committed context length
        self.pending = int(pending)   # the token verified last (position t_pos), key of the next query
        self.committed: List[int] = []  # tokens the target has committed behind the prompt (draft absorbs them)
        self.emitted: List[int] = [int(pending)]
        self.d_ctx = ctx_len          # draft: committed context length
        self.d_absorbed = 0
        self.stop = False
        self.error: Optional[BaseException] = None
        self.stats: Dict[str, float] = {"steps": 0, "hits": 0, "levels": 0, "restarts": 0, "stale_writes": 0}

    # ---------------------------------------------------------------- target side
    def _target_loop(self, n_tokens: int, stream: torch.cuda.Stream) -> None:
        tgt, r_max = self.tgt, self.depth + 1
        with torch.cuda.stream(stream):
            while len(self.emitted) - 1 < n_tokens and not self.stop:
                if self.wait_levels > 0:
                    t_end = time.perf_counter() + self.wait_ms * 1e-3
                    while self.cache.depth() < self.wait_levels + 1 and time.perf_counter() < t_end and not self.error:
                        time.sleep(0.0001)
                hit, path, _ = self.cache.query(self.pending, r_max)
                cand = path if hit else [self.pending]
                res = tgt.verify(self.t_pos, self.pending, cand)
                a = res["accepted_len"]
                if a < 1:
                    raise RuntimeError(f"target step failed: {res}")
                with self.lock:
                    self.cache.correct(cand[:a])
                    self.committed += cand[:a]
                    self.t_pos += a
                    self.pending = res["correction_token"]
                    self.emitted += cand[1:a] + [self.pending]
                self.stats["steps"] += 1
                self.stats["hits"] += int(hit)

    # ---------------------------------------------------------------- draft side
    def _draft_loop(self, stream: torch.cuda.Stream) -> None:
        dr, K, k = self.dr, self.K, self.k
        dev = dr.device
        with torch.cuda.stream(stream):
            while not self.stop:
                with self.lock:
                    new = list(self.committed[self.d_absorbed:])
                    root, epoch = self.pending, self.cache.epoch()
                    root_index = len(self.emitted) - 1  # text index of the root token
                # The draft's own cache has to hold everything in front of the root.  The tokens the
                # target has committed since the last tree are forwarded in the same call as the root
                # (a chain in front of it), whatever does not fit in front of that call on its own.
                max_r = dr.cfg.max_r
                while len(new) > max_r - 1:
                    chunk = new[: max_r - 1]
                    dr.verify(self.d_ctx, -1, chunk)
                    self.d_ctx += len(chunk)
                    self.d_absorbed += len(chunk)
                    new = new[len(chunk):]
                ctx_len = self.d_ctx                      # context the draft's cache holds already
                n_new = len(new)
                root_pos = ctx_len + n_new                # position and slot of the root token
                mask_base = ctx_len // 16 * 16
                words = (root_pos + 1 + K * self.depth - mask_base + 31) // 32
                if words > 32 or root_pos + 1 + K * self.depth > dr.cfg.max_ctx:
                    raise RuntimeError("draft cache too small for the tree")
                if self.cache.write(0, [root], [-1], [1.0], epoch=epoch) != B.CARD_OK:
                    self.stats["stale_writes"] += 1
                    continue
                self.stats["restarts"] += 1
                # mask rows of the chain [committed tokens ..., root]: each sees the one before it
                chain, prev_row = [], None
                for i in range(n_new + 1):
                    st, row = B.card_tree_mask_level(prev_row, [-1 if i == 0 else 0], ctx_len + i, ctx_len, mask_base, words)
                    chain.append(row[0])
                    prev_row = row
                toks, rows, first = list(new) + [root], chain, ctx_len
                positions = [ctx_len + i for i in range(n_new + 1)]
                sigma = torch.ones(1, dtype=torch.float32, device=dev)
                skip = n_new  # rows of the first call that are context, not tree nodes
                for l in range(self.depth):
                    res = dr.draft_level(ctx_len, toks, positions, first, rows, mask_base, k)
                    n_par = len(toks) - skip
                    ot = torch.empty(K, dtype=torch.int32, device=dev)
                    os_ = torch.empty(K, dtype=torch.float32, device=dev)
                    op = torch.empty(K, dtype=torch.int32, device=dev)
                    cnt = B.card_cache_select(sigma, res["topk_tokens"][skip:], res["topk_probs"][skip:], n_par, k, K, ot,
                                              os_, op, stream.cuda_stream)
                    if cnt < 0:
                        raise B.CardError(cnt, "card_cache_select")
                    stream.synchronize()
                    nt, npar, ns = ot[:cnt].tolist(), op[:cnt].tolist(), os_[:cnt].tolist()
                    if self.plant is not None:
                        nt, npar = self.plant(root_index + l + 1, l + 1, nt, npar)
                    if l == 0:
                        # the committed tokens are in the draft's cache from here on, whatever happens to the tree
                        self.d_ctx += n_new
                        self.d_absorbed += n_new
                    if self.stop or self.cache.write(l + 1, nt, npar, ns, epoch=epoch) != B.CARD_OK:
                        self.stats["stale_writes"] += 1
                        break  # the target has corrected the cache meanwhile: start again below its new token
                    self.stats["levels"] += 1
                    first += len(toks)
                    st, rows = B.card_tree_mask_level(rows[skip:], npar, first, ctx_len, mask_base, words)
                    toks, sigma, skip = nt, os_[:cnt].clone(), 0
                    positions = [root_pos + l + 1] * len(toks)
                else:
                    # the tree is as deep as it gets: wait for the target's next correction
                    while not self.stop and self.cache.epoch() == epoch:
                        time.sleep(0.0002)

    # ---------------------------------------------------------------- run
    def run(self, n_tokens: int) -> Dict[str, float]:
        s_t, s_d = _loop_streams(self.tgt.device)

        def guard(fn, *args):
            try:
                fn(*args)
            except BaseException as e:  # noqa: BLE001  (reported by run())
                self.error = e
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
                "stale_writes": self.stats["stale_writes"], "ms_per_target_step": dt * 1e3 / steps}
