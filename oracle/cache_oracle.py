"""CPU oracle for CARD's shared candidate cache: construction of one level, query, correction.

TEST INFRASTRUCTURE ONLY (see card_oracle.py); shares no code with the library.

The cache is the tree the draft model grows and the target model reads (Cache
Construction; Cache Correction).  Level l of the tree is the primary cache
C^(l): at most K nodes, each the last token of one length-(l+1) sequence, with
the index of its parent in level l-1 and its path score.  Level 0 holds the
candidates for the next position the target has not verified yet.

Readings where the text leaves room (each also listed in the design notes):
  * query: the key is the token the target has just verified.  A hit is a
    level-0 node carrying that token (the one with the largest score if there
    are several, the lowest index among equals).  The returned path starts
    with that token and follows parent links down to the best-scoring
    descendant on the deepest level that still has one (Fig. 2: "selects the
    highest-confidence path"; CARD Design: "highest-weighted candidate token
    sequence").
  * correct: the verified tokens are walked down from level 0; the children
    of the last matched node become the new level 0 and everything outside
    that subtree is dropped (Cache Correction: entries on wrong paths are
    pruned; siblings that were kept let a later query hit even after a
    rejection).  A verified token with no node empties the cache.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- eqs (1)-(9)


def build_level(
    probs: np.ndarray, sigma: np.ndarray, K: int, k: int
) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One layer of cache construction from the draft's next-token distributions.

    probs [K_in, V]: P_i of eq. (1); sigma [K_in]: cumulative probability of parent i,
    eq. (4).  Per parent take the top-k tokens (eq. 2), score each w = p * sigma (eq. 3),
    pool the K_in*k tuples (token, w, parent) (eq. 5), sort by score descending (eq. 6)
    and keep the first K (eq. 7).  Returns (tokens, scores, parents) of the new level;
    appending token m to parent m's sequence gives eqs. (8)-(9).  Equal scores are ordered
    by (parent, token) ascending so the result is unique."""
    k_in, vocab = probs.shape
    pool = []
    for i in range(k_in):
        order = sorted(range(vocab), key=lambda t: (-probs[i, t], t))[:k]
        for t in order:
            pool.append((float(probs[i, t]) * float(sigma[i]), i, t))
    pool.sort(key=lambda e: (-e[0], e[1], e[2]))
    pool = pool[:K]
    toks = np.array([e[2] for e in pool], dtype=np.int32)
    scores = np.array([e[0] for e in pool], dtype=np.float64)
    parents = np.array([e[1] for e in pool], dtype=np.int32)
    return toks, scores, parents


def tree_mask(parents_per_level: Sequence[Sequence[int]]) -> np.ndarray:
    """Draft attention mask over all tree nodes (Mask Construction for Draft Model).
    Node order: level by level.  Row of a node = its parent's row (inherited causal history)
    plus itself; peers of one level never see each other."""
    offs = np.cumsum([0] + [len(p) for p in parents_per_level])
    n = int(offs[-1])
    m = np.zeros((n, n), dtype=bool)
    for lvl, parents in enumerate(parents_per_level):
        for i, p in enumerate(parents):
            row = offs[lvl] + i
            if lvl > 0:
                m[row] = m[offs[lvl - 1] + p]
            m[row, row] = True
    return m


# --------------------------------------------------------------------------- tree with query / correct


@dataclass
class Level:
    tokens: List[int] = field(default_factory=list)
    parents: List[int] = field(default_factory=list)
    scores: List[float] = field(default_factory=list)


class CandidateCacheOracle:
    def __init__(self, K: int, max_depth: int):
        self.K = K
        self.max_depth = max_depth
        self.levels: List[Level] = []
        self.epoch = 0

    def depth(self) -> int:
        return len(self.levels)

    def write_level(self, level: int, tokens, parents, scores) -> None:
        """Store level `level` (0 = candidates for the next unverified position).  Level l
        needs level l-1 to exist; writing an existing level replaces it and drops deeper ones."""
        n = len(tokens)
        assert 0 <= level <= len(self.levels) and level < self.max_depth and 0 < n <= self.K
        if level == 0:
            assert all(p == -1 for p in parents)
        else:
            assert all(0 <= p < len(self.levels[level - 1].tokens) for p in parents)
        del self.levels[level:]
        self.levels.append(Level([int(t) for t in tokens], [int(p) for p in parents], [float(s) for s in scores]))

    def _match(self, level: int, token: int, parent: Optional[int]) -> int:
        lv = self.levels[level]
        best = -1
        for i, t in enumerate(lv.tokens):
            if t != token:
                continue
            if parent is not None and lv.parents[i] != parent:
                continue
            if best < 0 or lv.scores[i] > lv.scores[best]:
                best = i
        return best

    def query(self, verified_token: int, max_len: int) -> Tuple[bool, List[int], float]:
        if not self.levels or max_len < 1:
            return False, [], 0.0
        root = self._match(0, verified_token, None)
        if root < 0:
            return False, [], 0.0
        # descendants of root, level by level
        alive = [{root}]
        for l in range(1, len(self.levels)):
            nxt = {i for i, p in enumerate(self.levels[l].parents) if p in alive[-1]}
            if not nxt:
                break
            alive.append(nxt)
        deepest = min(len(alive), max_len) - 1
        lv = self.levels[deepest]
        leaf = min(alive[deepest], key=lambda i: (-lv.scores[i], i))
        score = lv.scores[leaf]
        path = []
        node = leaf
        for l in range(deepest, -1, -1):
            path.append(self.levels[l].tokens[node])
            node = self.levels[l].parents[node]
        path.reverse()
        return True, path, score

    def correct(self, verified_tokens: Sequence[int]) -> bool:
        """Re-root below the verified chain.  Returns False (and empties the cache) when the
        chain leaves the tree."""
        self.epoch += 1
        node = None
        for depth, tok in enumerate(verified_tokens):
            if depth >= len(self.levels):
                self.levels = []
                return False
            node = self._match(depth, int(tok), node)
            if node < 0:
                self.levels = []
                return False
        n = len(verified_tokens)
        if n == 0:
            return True
        keep = {node}
        new_levels: List[Level] = []
        for l in range(n, len(self.levels)):
            lv = self.levels[l]
            idx = [i for i, p in enumerate(lv.parents) if p in keep]
            if not idx:
                break
            remap = {old: new for new, old in enumerate(sorted(keep))}
            new_levels.append(
                Level(
                    [lv.tokens[i] for i in idx],
                    [-1 if l == n else remap[lv.parents[i]] for i in idx],
                    [lv.scores[i] for i in idx],
                )
            )
            keep = set(idx)
        self.levels = new_levels
        return True
