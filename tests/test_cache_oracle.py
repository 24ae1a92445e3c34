"""Pins of the shared-cache oracle (CPU only): the worked three-step example of the paper's
overview figure, eqs. (1)-(9) by brute force, and the two mask rules."""
import itertools

import numpy as np

from oracle.cache_oracle import CandidateCacheOracle, build_level, tree_mask

# word -> arbitrary id (the words are the ones used in the overview figure's caption)
W = {w: i + 10 for i, w in enumerate(
    ["Card", "was", "no", "ordinary", "souvenir", "-", "piece", "of", "paper", ",", "it", "sparkled",
     "is", "a", "the", "gift"])}


def _fig2_tree():
    """A tree that contains the caption's paths: Card -> was -> no -> ordinary -> {souvenir -> '-',
    piece -> of -> paper -> ',' -> it}, plus lower-scored distractors."""
    c = CandidateCacheOracle(K=8, max_depth=9)
    c.write_level(0, [W["Card"], W["gift"]], [-1, -1], [0.9, 0.1])
    c.write_level(1, [W["was"], W["is"]], [0, 0], [0.7, 0.2])
    c.write_level(2, [W["no"], W["a"]], [0, 1], [0.6, 0.1])
    c.write_level(3, [W["ordinary"], W["the"]], [0, 0], [0.5, 0.05])
    c.write_level(4, [W["souvenir"], W["piece"]], [0, 0], [0.30, 0.15])
    c.write_level(5, [W["-"], W["of"]], [0, 1], [0.25, 0.12])
    c.write_level(6, [W["paper"]], [1], [0.10])
    c.write_level(7, [W[","]], [0], [0.08])
    c.write_level(8, [W["it"]], [0], [0.07])
    return c


def _fake_target(prefix_words):
    """Lookup-table target: the text the target itself would write."""
    truth = ["Card", "was", "no", "ordinary", "piece", "of", "paper", ",", "it", "sparkled"]
    assert prefix_words == truth[: len(prefix_words)]
    return truth[len(prefix_words)]


def _accept(path_words, verified_so_far):
    """Greedy acceptance of a path whose first word is the already verified token."""
    acc = 1
    while acc < len(path_words) and _fake_target(verified_so_far + path_words[1:acc]) == path_words[acc]:
        acc += 1
    nxt = _fake_target(verified_so_far + path_words[1:acc])
    return acc, nxt


def test_overview_figure_three_steps():
    inv = {v: k for k, v in W.items()}
    c = _fig2_tree()
    # step 1: the communication ratio of the figure is 3, so a path carries the key + 2 tokens
    hit, path, _ = c.query(W["Card"], 3)
    words = [inv[t] for t in path]
    assert hit and words == ["Card", "was", "no"]
    acc, nxt = _accept(words, ["Card"])
    assert (acc, nxt) == (3, "ordinary")  # "was no" accepted, "ordinary" sampled
    assert c.correct([W[w] for w in words[:acc]])
    # step 2: hit on "ordinary", best path "souvenir -" is rejected at its first token
    hit, path, _ = c.query(W["ordinary"], 3)
    words = [inv[t] for t in path]
    assert hit and words == ["ordinary", "souvenir", "-"]
    acc, nxt = _accept(words, ["Card", "was", "no", "ordinary"])
    assert (acc, nxt) == (1, "piece")
    assert c.correct([W["ordinary"]])
    # step 3: the sibling kept in the cache still gives a hit after the rejection
    hit, path, _ = c.query(W["piece"], 5)
    words = [inv[t] for t in path]
    assert hit and words == ["piece", "of", "paper", ",", "it"]
    acc, nxt = _accept(words, ["Card", "was", "no", "ordinary", "piece"])
    assert (acc, nxt) == (5, "sparkled")
    assert c.correct([W[w] for w in words])
    assert c.depth() == 0  # nothing below "it" was drafted yet
    assert c.query(W["sparkled"], 3)[0] is False  # miss -> plain decode step


def test_query_miss_and_correct_off_tree_empties_cache():
    c = _fig2_tree()
    assert c.query(W["paper"], 4) == (False, [], 0.0)  # present deeper, but not at level 0
    assert c.correct([W["Card"], W["sparkled"]]) is False
    assert c.depth() == 0


def test_query_prefers_best_leaf_on_deepest_level_and_truncates():
    c = CandidateCacheOracle(K=4, max_depth=4)
    c.write_level(0, [5, 6], [-1, -1], [0.6, 0.4])
    c.write_level(1, [7, 8, 9], [0, 0, 1], [0.30, 0.25, 0.2])
    c.write_level(2, [1, 2], [1, 1], [0.10, 0.20])  # only node "8" has children
    assert c.query(5, 8) == (True, [5, 8, 2], 0.20)
    assert c.query(5, 2) == (True, [5, 7], 0.30)  # truncated: best node of level 1 under 5
    assert c.query(6, 8) == (True, [6, 9], 0.2)
    assert c.query(5, 1) == (True, [5], 0.6)


def test_correct_reindexes_parents():
    c = CandidateCacheOracle(K=4, max_depth=4)
    c.write_level(0, [5, 6], [-1, -1], [0.6, 0.4])
    c.write_level(1, [7, 8, 9], [0, 1, 1], [0.30, 0.25, 0.2])
    c.write_level(2, [1, 2, 3], [0, 1, 2], [0.10, 0.20, 0.15])
    assert c.correct([6])
    assert [(l.tokens, l.parents) for l in c.levels] == [([8, 9], [-1, -1]), ([2, 3], [0, 1])]
    assert c.epoch == 1


def test_build_level_bruteforce():
    rng = np.random.default_rng(0)
    for K_in, V, K, k in [(3, 7, 4, 2), (4, 9, 6, 3), (2, 5, 10, 5), (5, 6, 3, 1)]:
        logits = rng.normal(size=(K_in, V))
        probs = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
        sigma = rng.uniform(0.05, 1.0, size=K_in)
        toks, scores, parents = build_level(probs, sigma, K, k)
        # brute force: a pair (i, t) survives iff fewer than k tokens beat it within parent i and
        # fewer than K surviving pairs beat it overall
        w = probs * sigma[:, None]
        in_topk = np.array([[np.sum(probs[i] > probs[i, t]) < k for t in range(V)] for i in range(K_in)])
        pairs = [(i, t) for i, t in itertools.product(range(K_in), range(V)) if in_topk[i, t]]
        keep = {(i, t) for (i, t) in pairs if sum(w[a, b] > w[i, t] for (a, b) in pairs) < K}
        assert set(zip(parents.tolist(), toks.tolist())) == keep
        assert len(toks) == min(K, K_in * k)
        assert np.all(np.diff(scores) <= 0)
        np.testing.assert_allclose(scores, [w[i, t] for i, t in zip(parents, toks)])


def test_build_level_two_layers_gives_path_products():
    # sigma of a level-2 sequence is the product of its conditional probabilities (eq. 4)
    p0 = np.array([[0.5, 0.3, 0.2]])
    t0, s0, par0 = build_level(p0, np.array([1.0]), K=2, k=2)
    assert t0.tolist() == [0, 1] and par0.tolist() == [0, 0]
    p1 = np.array([[0.1, 0.6, 0.3], [0.7, 0.2, 0.1]])
    t1, s1, par1 = build_level(p1, s0, K=3, k=2)
    assert list(zip(par1.tolist(), t1.tolist())) == [(0, 1), (1, 0), (0, 2)]
    np.testing.assert_allclose(s1, [0.5 * 0.6, 0.3 * 0.7, 0.5 * 0.3])


def test_tree_mask_rules():
    parents = [[-1, -1], [0, 0, 1], [2, 0]]
    m = tree_mask(parents)
    n = m.shape[0]
    assert n == 7 and np.all(np.diag(m))
    # peers never see each other
    for lo, hi in [(0, 2), (2, 5), (5, 7)]:
        blk = m[lo:hi, lo:hi]
        assert np.array_equal(blk, np.eye(hi - lo, dtype=bool))
    # a node sees exactly its ancestors and itself
    assert np.flatnonzero(m[5]).tolist() == [1, 4, 5]
    assert np.flatnonzero(m[6]).tolist() == [0, 2, 6]
    assert not np.any(np.triu(m, 1))
