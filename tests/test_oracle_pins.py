"""Pins of the verify-step oracle against things other than itself (CPU only).

Each test names the mistake it is there to catch.  What fixes the expected values:
mathematics (closed forms, invariances), torch's CPU library routines used as
independent implementations of the textbook blocks, brute-force autoregressive
decoding, and the planted-prefix invariant of greedy verification (CARD Design:
verification is lossless; Fig. 2: accept the matching prefix, then emit the
target's own token).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import card_inputs as ci
from oracle import card_oracle as co
from oracle.from_inputs import oracle_weights

TINY = ci.SHAPES["tiny"]
# a shape with every dimension distinct and G = 3, so that swapped axes cannot cancel
ODD = ci.ModelShape("odd", 3, 96, 6, 2, 16, 80, 211, rope_theta=100.0, ctx=9, r=5)


def _rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------- blocks


def test_rmsnorm_matches_torch_and_unit_rms():
    x = _rng(0).normal(size=(5, 96)) * 3.0
    g = 1.0 + 0.3 * _rng(1).normal(size=96)
    got = co.rmsnorm(x, g, 1e-5)
    ref = F.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    unit = co.rmsnorm(x, np.ones(96), 0.0)
    np.testing.assert_allclose(np.sqrt((unit**2).mean(-1)), 1.0, rtol=1e-12)


def test_silu_matches_torch():
    z = np.linspace(-12, 12, 101)
    np.testing.assert_allclose(co.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-12, atol=1e-15)


def test_softmax_sums_to_one_and_shift_invariant():
    s = _rng(2).normal(size=37) * 5
    p = co.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-14
    np.testing.assert_allclose(co.softmax(s + 1000.0), p, rtol=1e-9)
    np.testing.assert_allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), rtol=1e-12)


def test_rope_closed_form_two_dims():
    # h = 2: a single pair turned by the angle pos * theta^0 = pos
    z = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -3.0]])
    out = co.rope(z, 3, 10000.0)
    c, s = math.cos(3.0), math.sin(3.0)
    np.testing.assert_allclose(out, [[c, s], [-s, c], [2 * c + 3 * s, -3 * c + 2 * s]], atol=1e-15)


def test_rope_is_complex_rotation_with_half_split_pairs():
    # wrong pairing (interleaved), wrong frequency exponent or a sign slip all fail here
    h, theta, pos = 16, 100.0, 7
    z = _rng(3).normal(size=(4, h))
    zc = torch.complex(torch.from_numpy(z[:, : h // 2]), torch.from_numpy(z[:, h // 2 :]))
    freqs = torch.tensor([theta ** (-(2 * j) / h) for j in range(h // 2)], dtype=torch.float64)
    rot = zc * torch.polar(torch.ones(h // 2, dtype=torch.float64), pos * freqs)
    ref = torch.cat([rot.real, rot.imag], -1).numpy()
    np.testing.assert_allclose(co.rope(z, pos, theta), ref, atol=1e-13)


def test_rope_identities():
    h = 32
    q, k = _rng(4).normal(size=h), _rng(5).normal(size=h)
    np.testing.assert_array_equal(co.rope(q, 0, 1e4), q)
    np.testing.assert_allclose(np.linalg.norm(co.rope(q, 123, 1e4)), np.linalg.norm(q), rtol=1e-13)
    a = co.rope(q, 50, 1e4) @ co.rope(k, 41, 1e4)
    b = co.rope(q, 1009, 1e4) @ co.rope(k, 1000, 1e4)
    assert abs(a - b) < 1e-10  # depends on the position difference only


def test_attend_row_matches_torch_sdpa_gqa():
    cfg = ODD
    hq, hkv, h, p = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 11
    q = _rng(6).normal(size=(hq, h))
    k = _rng(7).normal(size=(p, hkv, h))
    v = _rng(8).normal(size=(p, hkv, h))
    got = co.attend_row(cfg, q, k, v)
    tq = torch.from_numpy(q)[None, :, None, :]  # [B, Hq, 1, h]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None]  # [B, Hkv, p, h]
    tv = torch.from_numpy(v).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, enable_gqa=True)[0, :, 0, :].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------- whole forward


def _torch_forward(cfg, w, tokens, store="exact"):
    """The decoder written with torch library routines only (embedding, rms_norm, linear,
    complex multiply for the rotation, scaled_dot_product_attention with is_causal and
    enable_gqa, silu) in fp64.  With store == "bf16", K (after rotation) and V pass through
    torch's own bfloat16 cast on their way into attention, as a bf16 cache would hold them."""
    cached = (lambda z: z.float().bfloat16().double()) if store == "bf16" else (lambda z: z)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    n, hq, hkv, h = len(tokens), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    x = F.embedding(torch.tensor(tokens, dtype=torch.long), t(w.embed))
    freqs = torch.tensor([cfg.rope_theta ** (-(2 * j) / h) for j in range(h // 2)], dtype=torch.float64)
    ph = torch.polar(torch.ones(n, h // 2, dtype=torch.float64), torch.arange(n, dtype=torch.float64)[:, None] * freqs)

    def rot(z):  # [n, H, h]
        zc = torch.complex(z[..., : h // 2], z[..., h // 2 :]) * ph[:, None, :]
        return torch.cat([zc.real, zc.imag], -1)

    for l in range(cfg.n_layers):
        wl = w.layer(l)
        u = F.rms_norm(x, (cfg.d_model,), t(wl["g_attn"]), cfg.rms_eps)
        q = rot(F.linear(u, t(wl["wq"])).view(n, hq, h)).transpose(0, 1)[None]
        k = cached(rot(F.linear(u, t(wl["wk"])).view(n, hkv, h))).transpose(0, 1)[None]
        v = cached(F.linear(u, t(wl["wv"]))).view(n, hkv, h).transpose(0, 1)[None]
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
        x = x + F.linear(o[0].transpose(0, 1).reshape(n, hq * h), t(wl["wo"]))
        u2 = F.rms_norm(x, (cfg.d_model,), t(wl["g_ffn"]), cfg.rms_eps)
        x = x + F.linear(F.silu(F.linear(u2, t(wl["wg"]))) * F.linear(u2, t(wl["wu"])), t(wl["wd"]))
    return F.linear(F.rms_norm(x, (cfg.d_model,), t(w.g_final), cfg.rms_eps), t(w.lm_head)).numpy()


@pytest.mark.parametrize("store", ["exact", "bf16"])
@pytest.mark.parametrize("cfg", [ODD, TINY.with_layers(1)], ids=["odd", "tiny1"])
def test_forward_matches_torch_library_composition(cfg, store):
    # "exact": the textbook decoder; "bf16": the same with the cache's rounding, done by torch's cast
    w = oracle_weights(cfg, 11, gain_jitter=0.3)
    toks = ci.uniform_tokens(11, "ctx_tokens", 0, 14, cfg.vocab).tolist()
    ref = _torch_forward(cfg, w, toks, store)
    kv = co.OracleKV.empty(cfg, 16, store=store)
    got = co.forward_rows(cfg, w, kv, toks, 0)
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(co.full_recompute(cfg, w, toks, store=store), ref, rtol=1e-9, atol=1e-11)
    if store == "bf16":  # the rounding is not a no-op: the two readings differ well above the tolerance
        assert np.abs(ref - _torch_forward(cfg, w, toks, "exact")).max() > 1e-5


def test_round_bf16_is_the_library_cast_ties_to_even():
    rng = _rng(21)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, size=4000),
                        # exact ties between neighbouring bf16 values, both parities, both signs
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), -(2.0 + 3 * 2.0 ** -7), 0.0, 1.0, -0.375]])
    for dt in (np.float64, np.float32):
        ref = torch.from_numpy(x.astype(np.float32)).bfloat16().double().numpy()
        got = co.round_bf16(x.astype(dt))
        assert got.dtype == dt
        np.testing.assert_array_equal(got.astype(np.float64), ref)
    assert co.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0  # tie -> even mantissa
    assert co.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    x2 = rng.normal(size=(3, 5))
    assert co.cache_value(x2, "exact") is x2
    with pytest.raises(ValueError):
        co.cache_value(x2, "fp8")


@pytest.mark.parametrize("store", ["bf16", "exact"])
def test_verify_equals_stepwise_decode_equals_full_recompute(store):
    cfg = ODD
    w = oracle_weights(cfg, 5, gain_jitter=0.3)
    ctx = ci.uniform_tokens(5, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    cand = ci.uniform_tokens(5, "cand_tokens", 0, cfg.r, cfg.vocab).tolist()
    kv_a = co.OracleKV.empty(cfg, 32, store=store)
    co.prefill(cfg, w, kv_a, ctx, chunk=4)
    batched = co.forward_rows(cfg, w, kv_a, cand, cfg.ctx)
    kv_b = co.OracleKV.empty(cfg, 32, store=store)
    co.prefill(cfg, w, kv_b, ctx, chunk=9)
    step = np.stack([co.forward_rows(cfg, w, kv_b, [c], cfg.ctx + i)[0] for i, c in enumerate(cand)])
    full = co.full_recompute(cfg, w, ctx + cand, store=store)[cfg.ctx :]
    np.testing.assert_allclose(batched, step, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(batched, full, rtol=1e-10, atol=1e-12)
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(kv_a.k[l][: cfg.ctx + cfg.r], kv_b.k[l][: cfg.ctx + cfg.r], atol=1e-12)


def test_float32_oracle_close_to_float64():
    cfg = TINY
    w64 = oracle_weights(cfg, 2)
    w32 = oracle_weights(cfg, 2, dtype=np.float32)
    toks = ci.uniform_tokens(2, "ctx_tokens", 0, 40, cfg.vocab).tolist()
    # unrounded cache: a bf16 store would turn the few-ulp difference of the two precisions into
    # whole bf16 steps on the elements that sit next to a rounding boundary
    a = co.forward_rows(cfg, w64, co.OracleKV.empty(cfg, 40, store="exact"), toks, 0)
    b = co.forward_rows(cfg, w32, co.OracleKV.empty(cfg, 40, np.float32, store="exact"), toks, 0, np.float32)
    assert b.dtype == np.float32
    assert np.abs(a - b).max() < 2e-5 * np.abs(a).max()


def test_gqa_equals_mha_with_repeated_kv_heads():
    cfg = ODD
    w = oracle_weights(cfg, 7)
    g = cfg.n_q_heads // cfg.n_kv_heads
    mha = ci.ModelShape("mha", cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_q_heads, cfg.head_dim,
                        cfg.d_ffn, cfg.vocab, rope_theta=cfg.rope_theta)

    def layer(l):
        wl = dict(w.layer(l))
        for name in ("wk", "wv"):
            m = wl[name].reshape(cfg.n_kv_heads, cfg.head_dim, cfg.d_model)
            wl[name] = np.repeat(m, g, axis=0).reshape(-1, cfg.d_model)
        return wl

    w2 = co.OracleWeights(w.embed, w.lm_head, w.g_final, layer)
    toks = ci.uniform_tokens(7, "ctx_tokens", 0, 8, cfg.vocab).tolist()
    a = co.forward_rows(cfg, w, co.OracleKV.empty(cfg, 8), toks, 0)
    b = co.forward_rows(mha, w2, co.OracleKV.empty(mha, 8), toks, 0)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)


def test_zero_gate_kills_ffn_and_vocab_permutation_permutes_argmax():
    cfg = ODD.with_layers(1)
    w = oracle_weights(cfg, 9)
    toks = ci.uniform_tokens(9, "ctx_tokens", 0, 6, cfg.vocab).tolist()
    base = co.forward_rows(cfg, w, co.OracleKV.empty(cfg, 6), toks, 0)

    def layer_zero_gate(l):
        wl = dict(w.layer(l))
        wl["wg"] = np.zeros_like(wl["wg"])
        return wl

    def layer_zero_down(l):
        wl = dict(w.layer(l))
        wl["wd"] = np.zeros_like(wl["wd"])
        return wl

    a = co.forward_rows(cfg, co.OracleWeights(w.embed, w.lm_head, w.g_final, layer_zero_gate),
                        co.OracleKV.empty(cfg, 6), toks, 0)
    b = co.forward_rows(cfg, co.OracleWeights(w.embed, w.lm_head, w.g_final, layer_zero_down),
                        co.OracleKV.empty(cfg, 6), toks, 0)
    np.testing.assert_allclose(a, b, atol=1e-14)  # silu(0) * up == 0: both remove the FFN
    assert np.abs(a - base).max() > 1e-3
    perm = _rng(10).permutation(cfg.vocab)
    wp = co.OracleWeights(w.embed, w.lm_head[perm], w.g_final, w.layer)
    lp = co.forward_rows(cfg, wp, co.OracleKV.empty(cfg, 6), toks, 0)
    np.testing.assert_allclose(lp, base[:, perm], atol=1e-14)
    assert [perm[co.argmax_lowest(r)] for r in lp] == [co.argmax_lowest(r) for r in base]


def test_argmax_ties_take_lowest_index_and_gap():
    row = np.array([0.5, 2.0, -1.0, 2.0, 1.5])
    assert co.argmax_lowest(row) == 1
    assert co.top2_gap(row) == 0.0
    assert abs(co.top2_gap(np.array([0.1, 0.9, 0.4])) - 0.5) < 1e-15


# ----------------------------------------------------------------------------- acceptance


def test_greedy_accept_table():
    # pending g0 = 7; rows predict 8, 9, 10, 11 after candidates c0..c3
    am = [8, 9, 10, 11]
    assert co.greedy_accept(7, am, [7, 8, 9, 10]) == (4, 11)  # all accepted: next token is row 3's
    assert co.greedy_accept(7, am, [7, 8, 5, 10]) == (2, 9)  # rejected at index 2: replacement
    assert co.greedy_accept(7, am, [6, 8, 9, 10]) == (0, 7)  # first candidate is not the pending token
    assert co.greedy_accept(-1, am, [6, 8, 9, 10]) == (4, 11)  # no pending token: row 0 is trusted
    assert co.greedy_accept(7, am[:1], [7]) == (1, 8)  # r = 1 is a plain decode step


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_planted_prefix_invariant_and_bruteforce_stream(seed):
    cfg = ODD
    w = oracle_weights(cfg, seed, gain_jitter=0.2)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    r = cfg.r
    brute = co.greedy_decode_bruteforce(cfg, w, ctx, r + 1)  # g0..g_r without any KV cache
    for j in range(r + 1):
        kv = co.OracleKV.empty(cfg, 32)
        g0 = co.prefill(cfg, w, kv, ctx)
        assert g0 == brute[0]
        cand = ci.plant_candidates(brute, j, r, cfg.vocab, seed, stream=j)
        res = co.verify(cfg, w, kv, cfg.ctx, g0, cand)
        assert res.accepted_len == j
        assert res.correction_token == brute[j]
        assert (res.kv_first_slot, res.kv_count) == (cfg.ctx, j)


def test_chained_verify_reproduces_greedy_stream_for_any_candidate_quality():
    cfg = ODD
    w = oracle_weights(cfg, 4)
    ctx = ci.uniform_tokens(4, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    want = co.greedy_decode_bruteforce(cfg, w, ctx, 12)
    kv = co.OracleKV.empty(cfg, 64)
    pending = co.prefill(cfg, w, kv, ctx)
    n, emitted, step = cfg.ctx, [pending], 0
    while len(emitted) < 12:
        # candidates: the pending token, then a mix of right and wrong guesses
        guess = want[len(emitted) : len(emitted) + 3]
        cand = [pending] + [g if (step + i) % 3 else (g + 1) % cfg.vocab for i, g in enumerate(guess)]
        res = co.verify(cfg, w, kv, n, pending, cand)
        assert res.accepted_len >= 1
        emitted += cand[1 : res.accepted_len] + [res.correction_token]
        n += res.kv_count
        pending = res.correction_token
        step += 1
    assert emitted[:12] == want


@pytest.mark.parametrize("store", ["bf16", "exact"])
@pytest.mark.parametrize("seed", [3, 6])
def test_greedy_decode_cached_equals_bruteforce_and_its_gaps_are_the_recomputed_rows(store, seed):
    """The cached decoder writes the greedy stream and the gaps of every stored golden and of
    most GPU cases.  Pinned against the cache-free path: the stream equals brute-force decoding
    (whole sequence recomputed per token) and gap i is the top-1/top-2 distance of the row of
    `full_recompute` that predicts token i+1.  A shifted position, a stale cache row or a gap
    taken from the wrong row fails here."""
    cfg = ODD
    w = oracle_weights(cfg, seed, gain_jitter=0.2)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    n_new = 7
    kv = co.OracleKV.empty(cfg, 32, store=store)
    g0 = co.prefill(cfg, w, kv, ctx, chunk=4)
    toks, gaps = co.greedy_decode_cached(cfg, w, kv, cfg.ctx, g0, n_new)
    assert len(toks) == n_new + 1 and len(gaps) == n_new and toks[0] == g0
    assert toks == co.greedy_decode_bruteforce(cfg, w, ctx, n_new + 1, store=store)
    full = co.full_recompute(cfg, w, ctx + toks[:-1], store=store)
    for i in range(n_new):  # the row at position ctx + i was fed toks[i] and predicts toks[i + 1]
        row = full[cfg.ctx + i]
        assert co.argmax_lowest(row) == toks[i + 1]
        assert abs(co.top2_gap(row) - gaps[i]) < 1e-9
    # the cache now holds the stream's keys: a further row sees exactly the recomputed history
    nxt = co.forward_rows(cfg, w, kv, [toks[-1]], cfg.ctx + n_new)[0]
    ref = co.full_recompute(cfg, w, ctx + toks, store=store)[-1]
    np.testing.assert_allclose(nxt, ref, rtol=1e-10, atol=1e-12)



# ----------------------------------------------------------------------------- sampling (temperature > 0)


def test_mixer_and_uniforms_of_the_noise_generator():
    # the mixer against the generators' own copy of the published function, and its fixed point
    x = np.array([0, 1, 2, 0xDEADBEEF, 0xFFFFFFFF, 123456789], dtype=np.uint64)
    assert co._mix32(x).tolist() == [ci.generate._mix32_int(int(v)) for v in x]
    assert int(co._mix32(np.array([0], dtype=np.uint64))[0]) == 0
    g = co.gumbel_noise(7, 1000, 4096)
    u = np.exp(-np.exp(-g))
    k = u * 2 ** 24 - 0.5  # u = (k + 1/2) / 2^24 with integer k: strictly inside (0, 1)
    assert np.abs(k - np.round(k)).max() < 1e-6 and k.min() >= 0 and k.max() <= 2 ** 24 - 1
    # another position, another seed half, another token: another draw
    assert not np.array_equal(g, co.gumbel_noise(7, 1001, 4096))
    assert not np.array_equal(g, co.gumbel_noise(7 + (1 << 32), 1000, 4096))
    assert len(np.unique(g)) > 4000


def test_noise_is_standard_gumbel():
    g = np.concatenate([co.gumbel_noise(3, p, 2048) for p in range(200)])
    assert abs(g.mean() - 0.5772156649) < 0.01  # Euler-Mascheroni
    assert abs(g.var() - math.pi ** 2 / 6) < 0.03
    # CDF exp(-exp(-x)) at a few points
    for x in (-1.0, 0.0, 1.0, 3.0):
        assert abs((g <= x).mean() - math.exp(-math.exp(-x))) < 0.005


def test_draws_follow_the_softmax_and_acceptance_rate_is_p_of_the_candidate():
    """Chi-square of the draw frequencies against softmax(logits / T), and the probability that the
    draw equals a fixed candidate (= the acceptance probability of a point-mass proposal)."""
    rng = _rng(11)
    logits = rng.normal(size=12) * 1.5
    for temp in (1.0, 0.7):
        p = co.softmax(logits / temp)
        n = 40000
        draws = np.array([co.argmax_lowest(co.perturbed(logits, pos, temp, 99)) for pos in range(n)])
        counts = np.bincount(draws, minlength=12)
        chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
        assert chi2 < 40.0  # 11 degrees of freedom: 40 is beyond the 99.99 % point
        c = int(np.argsort(p)[-2])
        assert abs((draws == c).mean() - p[c]) < 4 * math.sqrt(p[c] * (1 - p[c]) / n)
    # temperature -> 0 is the arg-max; temperature 0 leaves the row untouched
    assert co.argmax_lowest(co.perturbed(logits, 5, 1e-4, 99)) == co.argmax_lowest(logits)
    assert co.perturbed(logits, 5, 0.0, 99) is logits


@pytest.mark.parametrize("seed", [2, 5])
def test_chained_sampled_verify_reproduces_token_by_token_sampling(seed):
    """Lossless at a temperature: whatever the candidates, chained verification steps emit exactly
    the text that plain autoregressive sampling with the same seed emits (cache-free recompute per
    token), and a planted prefix of that text is accepted to its full length."""
    cfg = ODD
    w = oracle_weights(cfg, seed, gain_jitter=0.2)
    ctx = ci.uniform_tokens(seed, "ctx_tokens", 0, cfg.ctx, cfg.vocab).tolist()
    temp, rs = 1.0, 1000 + seed
    want = co.greedy_decode_bruteforce(cfg, w, ctx, 12, temperature=temp, seed=rs)
    assert want != co.greedy_decode_bruteforce(cfg, w, ctx, 12)  # it is not the greedy text
    kv = co.OracleKV.empty(cfg, 64)
    last = co.forward_rows(cfg, w, kv, ctx, 0)[-1]
    pending = co.argmax_lowest(co.perturbed(last, cfg.ctx, temp, rs))
    assert pending == want[0]
    # planted prefixes of the sampled text
    for j in range(cfg.r + 1):
        cand = ci.plant_candidates(want, j, cfg.r, cfg.vocab, seed, stream=j)
        res = co.verify(cfg, w, kv, cfg.ctx, pending, cand, temperature=temp, seed=rs)
        assert (res.accepted_len, res.correction_token) == (j, want[j])
    n, emitted, step = cfg.ctx, [pending], 0
    while len(emitted) < 12:
        guess = want[len(emitted): len(emitted) + 3]
        cand = [pending] + [g if (step + i) % 3 else (g + 1) % cfg.vocab for i, g in enumerate(guess)]
        res = co.verify(cfg, w, kv, n, pending, cand, temperature=temp, seed=rs)
        emitted += cand[1: res.accepted_len] + [res.correction_token]
        n += res.kv_count
        pending = res.correction_token
        step += 1
    assert emitted[:12] == want
    toks, _ = co.greedy_decode_cached(cfg, w, co_kv_prefilled(cfg, w, ctx), cfg.ctx, want[0], 6, temperature=temp, seed=rs)
    assert toks == want[:7]


def co_kv_prefilled(cfg, w, ctx):
    kv = co.OracleKV.empty(cfg, 64)
    co.prefill(cfg, w, kv, ctx)
    return kv


def test_a_stored_full_size_case_is_accepted_in_full_with_every_row_decisive():
    """The bit-exact accept / correct criterion needs at least one full-size step whose r deciding
    rows all clear the 0.05 gap (a fully accepted r = 8 step): the stored goldens must hold one."""
    import glob
    import json
    import os

    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    found = []
    for path in sorted(glob.glob(os.path.join(root, "llama8b_seed*.json"))):
        with open(path) as f:
            g = json.load(f)
        assert g["kv_store"] == "bf16", path
        w = g.get("window")
        if w and w["accepted_len"] == g["r"] == 8 and all(gap > 0.05 for gap in w["row_gap"]):
            assert w["cand"][0] == w["pending"] and w["ctx_len"] == g["ctx"] + len(w["extra_ctx"])
            found.append(os.path.basename(path))
    assert found, "no stored full-size step with eight decisive rows"
