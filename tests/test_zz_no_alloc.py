"""The entry point that allocates nothing (card_verify_static: workspace = an array inside the
library's code object) against card_verify, through the C ABI: two calls in a row on the same
GPU, the second with a smaller input (fewer rows, shorter context, the cache rows of the first
call left in place), then a call for another model shape, which has to re-prepare the shared
array.  Integers bit-exact; the K and V rows each call writes are compared bit for bit as well
(both paths run the same kernel in the same order, so nothing may differ)."""
import pytest
import torch

import card_inputs as ci

pytestmark = pytest.mark.gpu

TINY = ci.SHAPES["tiny"]
MID = ci.ModelShape("mid", 3, 512, 8, 2, 128, 1048, 3001, ctx=200, r=8)


def _pair(shape, seed, max_ctx):
    import paper_2508_04462_amd as card
    from paper_2508_04462_amd.synthetic import load_synthetic_weights

    a = card.Target(shape, max_ctx)
    load_synthetic_weights(a, shape, seed, 0.2)
    b = card.Target(shape, max_ctx)
    b.packed.copy_(a.packed)
    return a, b


def _static_verify(tgt, ctx_len, pending, cand):
    import paper_2508_04462_amd as card

    r = len(cand)
    tgt.cand[:r] = torch.tensor(cand, dtype=torch.int32, device=tgt.device)
    tgt.out.fill_(-7)
    tgt.row_argmax.fill_(-7)
    st = card.card_verify_static(tgt.cfg, tgt.packed, tgt.kv(pending), ctx_len, tgt.cand, r, tgt._stream(), tgt.out,
                                 tgt.row_argmax)
    assert st == card.CARD_OK, card.card_strerror(st)
    torch.cuda.current_stream(tgt.device).synchronize()
    o = tgt.out.tolist()
    return {"accepted_len": o[0], "correction_token": o[1], "kv_first_slot": o[2], "kv_count": o[3],
            "row_argmax": tgt.row_argmax[:r].tolist()}


def _same_kv(a, b, shape, first, count):
    for l in range(shape.n_layers):
        ka, va = a.kv_gather(l, first, count)
        kb, vb = b.kv_gather(l, first, count)
        assert torch.equal(ka, kb) and torch.equal(va, vb), l


def _two_calls(shape, seed, ctx1, r1, ctx2, r2):
    a, b = _pair(shape, seed, 320)
    toks = ci.uniform_tokens(seed, "ctx_tokens", 0, ctx1 + r1, shape.vocab).tolist()
    g0a = a.prefill(toks[:ctx1])
    g0b = b.prefill(toks[:ctx1])
    assert g0a == g0b
    # first call: r1 rows at ctx1, the first candidate is the pending token (a CARD step)
    cand1 = [g0a] + toks[ctx1 + 1: ctx1 + r1]
    ref1 = a.verify(ctx1, g0a, cand1)
    got1 = _static_verify(b, ctx1, g0a, cand1)
    for k in got1:
        assert got1[k] == ref1[k], (k, got1[k], ref1[k])
    assert got1["accepted_len"] >= 1
    _same_kv(a, b, shape, ctx1, r1)
    # second call, smaller: fewer rows at a shorter context (rows beyond it stay from before)
    cand2 = toks[ctx2: ctx2 + r2]
    ref2 = a.verify(ctx2, -1, cand2)
    got2 = _static_verify(b, ctx2, -1, cand2)
    for k in got2:
        assert got2[k] == ref2[k], (k, got2[k], ref2[k])
    assert got2["accepted_len"] >= 1  # no pending token: the first candidate is taken as given
    _same_kv(a, b, shape, ctx2, r2)


def test_static_entry_point_matches_card_verify_on_two_calls_in_a_row():
    import paper_2508_04462_amd as card

    assert card.card_workspace_bytes(card.make_cfg(MID, 320)) <= card.card_static_scratch_bytes()
    _two_calls(MID, 21, ctx1=150, r1=8, ctx2=61, r2=3)
    # another model shape on the same GPU: the control words live elsewhere in the shared array
    _two_calls(TINY, 22, ctx1=100, r1=17, ctx2=33, r2=4)
    # and back, after an explicit reset
    assert card.card_static_scratch_reset() == card.CARD_OK
    _two_calls(MID, 23, ctx1=40, r1=5, ctx2=16, r2=1)


def test_static_entry_point_rejects_a_model_beyond_its_scratch():
    import paper_2508_04462_amd as card

    cfg = card.make_cfg(ci.SHAPES["llama8b"], 2048)
    assert card.card_workspace_bytes(cfg) > card.card_static_scratch_bytes()
    kv = card.CardKV(0x1000, 0x1000, 0x1000, 16, -1)
    st = card.card_verify_static(cfg, 0x1000, kv, 0, 0x1000, 1, None, 0x1000, None)
    assert st == card.CARD_ETOOBIG and "static scratch" in card.card_strerror(st)
