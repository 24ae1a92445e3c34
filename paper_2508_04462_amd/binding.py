"""ctypes binding of include/card.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_PKG, "libcard.so")

CARD_OK, CARD_EINVAL, CARD_ERANGE, CARD_ECAPACITY, CARD_EDEVICE, CARD_ESTALE, CARD_ETOOBIG = 0, -1, -2, -3, -4, -5, -6

TENSOR_IDS = {
    "embed": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "wg": 5, "wu": 6, "wd": 7,
    "lm_head": 8, "g_attn": 9, "g_ffn": 10, "g_final": 11,
}


class CardError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {card_strerror(status)} ({status})")


class CardModelCfg(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
        ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
        ("kv_block", C.c_int32), ("max_ctx", C.c_int32), ("max_r", C.c_int32), ("grid_wgs", C.c_int32),
    ]


class CardKV(C.Structure):
    _fields_ = [
        ("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("block_table", C.c_void_p),
        ("n_pages", C.c_int32), ("pending_token", C.c_int32),
    ]


class CardSampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("seed", C.c_uint64)]


class CardTreeRows(C.Structure):
    _fields_ = [("tokens_dev", C.c_void_p), ("positions_dev", C.c_void_p), ("first_slot", C.c_int32),
                ("mask_dev", C.c_void_p), ("mask_words", C.c_int32), ("mask_base", C.c_int32)]


class CardStep(C.Structure):
    _fields_ = [("r", C.c_int32), ("hit", C.c_int32), ("path_score", C.c_float), ("cand", C.c_int32 * 32)]


CARD_STEP_NO_CORRECT = 1


class CardVerifyResult(C.Structure):
    _fields_ = [
        ("accepted_len", C.c_int32), ("correction_token", C.c_int32),
        ("kv_first_slot", C.c_int32), ("kv_count", C.c_int32),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(lib_path):
        raise ImportError(
            f"{lib_path} is missing: build it with `python -m paper_2508_04462_amd.build` "
            "(there is no fallback path)")
    return C.CDLL(lib_path)


_P = C.c_void_p
_cfgp = C.POINTER(CardModelCfg)
_kvp = C.POINTER(CardKV)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


def _declare(lib: C.CDLL) -> C.CDLL:
    """Result and argument types of every entry point of include/card.h."""
    lib.card_strerror.restype = C.c_char_p
    lib.card_strerror.argtypes = [C.c_int]
    for _n in ("card_packed_weight_bytes", "card_workspace_bytes"):
        getattr(lib, _n).restype = C.c_size_t
        getattr(lib, _n).argtypes = [_cfgp]
    lib.card_stream_frag_index.restype = C.c_int64
    lib.card_stream_frag_index.argtypes = [C.c_int32] * 6
    lib.card_kv_pool_bytes.restype = C.c_size_t
    lib.card_kv_pool_bytes.argtypes = [_cfgp, C.c_int32]
    lib.card_weights_pack_tensor.restype = C.c_int
    lib.card_weights_pack_tensor.argtypes = [_cfgp, C.c_int32, C.c_int32, _P, _P, _P]
    lib.card_workspace_init.restype = C.c_int
    lib.card_workspace_init.argtypes = [_cfgp, _P, _P]
    lib.card_verify.restype = C.c_int
    lib.card_verify.argtypes = [_cfgp, _P, _kvp, C.c_int32, _P, C.c_int32, _P, _P, _P, _P]
    lib.card_verify_sampled.restype = C.c_int
    lib.card_verify_sampled.argtypes = [_cfgp, _P, _kvp, C.c_int32, _P, C.c_int32, C.POINTER(CardSampling), _P, _P, _P, _P, _P]
    lib.card_draft_level.restype = C.c_int
    lib.card_draft_level.argtypes = [_cfgp, _P, _kvp, C.c_int32, C.POINTER(CardTreeRows), C.c_int32, C.c_int32, _P, _P, _P, _P, _P]
    lib.card_tree_mask_level.restype = C.c_int
    lib.card_tree_mask_level.argtypes = [_P, _i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P]
    lib.card_cache_select.restype = C.c_int
    lib.card_cache_select.argtypes = [_P, _P, _P, C.c_int32, C.c_int32, C.c_int32, _P, _P, _P, _P]
    lib.card_step_begin.restype = C.c_int
    lib.card_step_begin.argtypes = [_P, _cfgp, _P, _kvp, C.c_int32, C.c_int32, _P, _P, _P, _P, _P, C.POINTER(CardStep)]
    lib.card_step_begin_sampled.restype = C.c_int
    lib.card_step_begin_sampled.argtypes = [_P, _cfgp, _P, _kvp, C.c_int32, C.c_int32, _P, _P, _P, _P, _P, C.POINTER(CardStep),
                                            C.POINTER(CardSampling)]
    lib.card_step_end.restype = C.c_int
    lib.card_step_end.argtypes = [_P, C.POINTER(CardStep), _P, C.c_int32, _i32p, _i32p]
    lib.card_verify_static.restype = C.c_int
    lib.card_verify_static.argtypes = [_cfgp, _P, _kvp, C.c_int32, _P, C.c_int32, _P, _P, _P]
    lib.card_static_scratch_bytes.restype = C.c_size_t
    lib.card_static_scratch_bytes.argtypes = []
    lib.card_static_scratch_reset.restype = C.c_int
    lib.card_static_scratch_reset.argtypes = []
    lib.card_verify_debug_logits.restype = C.c_int
    lib.card_verify_debug_logits.argtypes = [_cfgp, _P, _kvp, C.c_int32, _P, C.c_int32, _P, _P, _P, _P, _P]
    lib.card_kv_gather.restype = C.c_int
    lib.card_kv_gather.argtypes = [_cfgp, _kvp, C.c_int32, C.c_int32, C.c_int32, _P, _P, _P]
    lib.card_profile_enable.restype = C.c_int
    lib.card_profile_enable.argtypes = [C.c_int32]
    lib.card_profile_disable.restype = C.c_int
    lib.card_profile_disable.argtypes = []
    lib.card_profile_timeline.restype = C.c_int
    lib.card_profile_timeline.argtypes = [_P, C.c_int32]
    lib.card_profile_collect.restype = C.c_int
    lib.card_profile_collect.argtypes = [_f32p, _i32p]
    lib.card_cache_create.restype = C.c_int
    lib.card_cache_create.argtypes = [C.c_int32, C.c_int32, C.POINTER(_P)]
    lib.card_cache_destroy.restype = None
    lib.card_cache_destroy.argtypes = [_P]
    lib.card_cache_write.restype = C.c_int
    lib.card_cache_write.argtypes = [_P, C.c_int64, C.c_int32, C.c_int32, _i32p, _i32p, _f32p]
    lib.card_cache_query.restype = C.c_int
    lib.card_cache_query.argtypes = [_P, C.c_int32, C.c_int32, _i32p, _i32p, _f32p]
    lib.card_cache_correct.restype = C.c_int
    lib.card_cache_correct.argtypes = [_P, _i32p, C.c_int32]
    lib.card_cache_epoch.restype = C.c_int64
    lib.card_cache_epoch.argtypes = [_P]
    lib.card_cache_depth.restype = C.c_int32
    lib.card_cache_depth.argtypes = [_P]
    lib.card_cache_read_level.restype = C.c_int
    lib.card_cache_read_level.argtypes = [_P, C.c_int32, _i32p, _i32p, _f32p]
    return lib


class _Library:
    """libcard.so, opened at the first use of any entry point (so that the build step can import
    this package before the library exists).  There is no other implementation behind it: a
    missing library raises ImportError at that first use."""

    def __init__(self):
        self._cdll = None

    def __getattr__(self, name):
        if self._cdll is None:
            self._cdll = _declare(_load())
        return getattr(self._cdll, name)


lib = _Library()


def _ptr(x) -> Optional[int]:
    """torch tensor -> its data pointer; int / None pass through."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def card_strerror(status: int) -> str:
    return lib.card_strerror(int(status)).decode()


def card_packed_weight_bytes(cfg: CardModelCfg) -> int:
    return lib.card_packed_weight_bytes(C.byref(cfg))


def card_workspace_bytes(cfg: CardModelCfg) -> int:
    return lib.card_workspace_bytes(C.byref(cfg))


def card_stream_frag_index(n_tiles: int, k_steps: int, batch: int, grid: int, t: int, s: int) -> int:
    return lib.card_stream_frag_index(n_tiles, k_steps, batch, grid, t, s)


def card_kv_pool_bytes(cfg: CardModelCfg, n_pages: int) -> int:
    return lib.card_kv_pool_bytes(C.byref(cfg), n_pages)


def card_weights_pack_tensor(cfg, tensor: int, layer: int, src_dev, packed_dev, stream=None) -> int:
    return lib.card_weights_pack_tensor(C.byref(cfg), tensor, layer, _ptr(src_dev), _ptr(packed_dev), _ptr(stream))


def card_verify(cfg, packed_dev, kv: CardKV, ctx_len: int, cand_dev, r: int, workspace_dev, stream,
                out_dev, row_argmax_dev=None) -> int:
    return lib.card_verify(C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, _ptr(cand_dev), r,
                           _ptr(workspace_dev), _ptr(stream), _ptr(out_dev), _ptr(row_argmax_dev))


def card_verify_sampled(cfg, packed_dev, kv: CardKV, ctx_len: int, cand_dev, r: int, sampling: CardSampling,
                        workspace_dev, stream, out_dev, row_token_dev=None, logits_dev=None) -> int:
    return lib.card_verify_sampled(C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, _ptr(cand_dev), r,
                                   C.byref(sampling), _ptr(workspace_dev), _ptr(stream), _ptr(out_dev),
                                   _ptr(row_token_dev), _ptr(logits_dev))


def card_draft_level(cfg, packed_dev, kv: CardKV, ctx_len: int, rows: CardTreeRows, n_rows: int, k: int,
                     workspace_dev, stream, topk_tokens_dev, topk_probs_dev, logits_dev=None) -> int:
    return lib.card_draft_level(C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, C.byref(rows), n_rows, k,
                                _ptr(workspace_dev), _ptr(stream), _ptr(topk_tokens_dev), _ptr(topk_probs_dev),
                                _ptr(logits_dev))


def card_tree_mask_level(parent_mask, parent_idx, first_slot: int, ctx_len: int, mask_base: int, mask_words: int):
    """parent_mask: list of rows (lists of mask_words uint32) or None; returns (status, rows)."""
    n = len(parent_idx)
    out = (C.c_uint32 * (n * mask_words))()
    pm = None
    if parent_mask is not None:
        flat = [int(w) for row in parent_mask for w in row]
        pm = (C.c_uint32 * len(flat))(*flat)
    st = lib.card_tree_mask_level(pm, _i32(parent_idx), n, first_slot, ctx_len, mask_base, mask_words, out)
    return st, [list(out[i * mask_words:(i + 1) * mask_words]) for i in range(n)]


def card_cache_select(sigma_dev, topk_tokens_dev, topk_probs_dev, n_parents: int, k: int, K: int, out_tokens_dev,
                      out_scores_dev, out_parents_dev, stream=None) -> int:
    return lib.card_cache_select(_ptr(sigma_dev), _ptr(topk_tokens_dev), _ptr(topk_probs_dev), n_parents, k, K,
                                 _ptr(out_tokens_dev), _ptr(out_scores_dev), _ptr(out_parents_dev), _ptr(stream))


def card_step_begin(cache, cfg, packed_dev, kv: CardKV, ctx_len: int, max_len: int, cand_staging, workspace_dev,
                    stream, out, row_argmax_dev, step: CardStep) -> int:
    return lib.card_step_begin(cache, C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, max_len,
                               _ptr(cand_staging), _ptr(workspace_dev), _ptr(stream), _ptr(out),
                               _ptr(row_argmax_dev), C.byref(step))


def card_step_begin_sampled(cache, cfg, packed_dev, kv: CardKV, ctx_len: int, max_len: int, cand_staging, workspace_dev,
                            stream, out, row_token_dev, step: CardStep, sampling: CardSampling) -> int:
    return lib.card_step_begin_sampled(cache, C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, max_len,
                                       _ptr(cand_staging), _ptr(workspace_dev), _ptr(stream), _ptr(out),
                                       _ptr(row_token_dev), C.byref(step), C.byref(sampling))


def card_step_end(cache, step: CardStep, out_host, flags: int = 0):
    """Returns (status, [emitted tokens])."""
    buf = (C.c_int32 * 33)()
    n = C.c_int32(0)
    st = lib.card_step_end(cache, C.byref(step), _ptr(out_host), flags, buf, C.byref(n))
    return st, list(buf[: n.value])


def card_verify_static(cfg, packed_dev, kv: CardKV, ctx_len: int, cand_dev, r: int, stream, out_dev,
                       row_argmax_dev=None) -> int:
    return lib.card_verify_static(C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, _ptr(cand_dev), r,
                                  _ptr(stream), _ptr(out_dev), _ptr(row_argmax_dev))


def card_static_scratch_bytes() -> int:
    return lib.card_static_scratch_bytes()


def card_static_scratch_reset() -> int:
    return lib.card_static_scratch_reset()


def card_verify_debug_logits(cfg, packed_dev, kv: CardKV, ctx_len: int, cand_dev, r: int, workspace_dev,
                             stream, out_dev, row_argmax_dev, logits_dev) -> int:
    return lib.card_verify_debug_logits(C.byref(cfg), _ptr(packed_dev), C.byref(kv), ctx_len, _ptr(cand_dev), r,
                                        _ptr(workspace_dev), _ptr(stream), _ptr(out_dev), _ptr(row_argmax_dev),
                                        _ptr(logits_dev))


def card_kv_gather(cfg, kv: CardKV, layer: int, first_slot: int, count: int, k_out_dev, v_out_dev,
                   stream=None) -> int:
    return lib.card_kv_gather(C.byref(cfg), C.byref(kv), layer, first_slot, count, _ptr(k_out_dev),
                              _ptr(v_out_dev), _ptr(stream))


def card_profile_enable(max_launches: int) -> int:
    return lib.card_profile_enable(max_launches)


def card_profile_disable() -> int:
    return lib.card_profile_disable()


def card_workspace_init(cfg, workspace_dev, stream=None) -> int:
    return lib.card_workspace_init(C.byref(cfg), _ptr(workspace_dev), _ptr(stream))


def card_profile_timeline(buf_dev, layer: int) -> int:
    return lib.card_profile_timeline(_ptr(buf_dev), layer)


def card_profile_collect(max_launches: int):
    """Returns (status, [ms per launch])."""
    buf = (C.c_float * max_launches)()
    n = C.c_int32(0)
    st = lib.card_profile_collect(buf, C.byref(n))
    return st, list(buf[: n.value])


def _i32(seq):
    return (C.c_int32 * len(seq))(*[int(v) for v in seq])


def card_cache_create(K: int, max_depth: int):
    h = _P()
    st = lib.card_cache_create(K, max_depth, C.byref(h))
    return st, h


def card_cache_destroy(handle) -> None:
    lib.card_cache_destroy(handle)


def card_cache_write(handle, epoch: int, level: int, tokens, parent_idx, path_score) -> int:
    n = len(tokens)
    sc = (C.c_float * n)(*[float(v) for v in path_score])
    return lib.card_cache_write(handle, epoch, level, n, _i32(tokens), _i32(parent_idx), sc)


def card_cache_query(handle, verified_token: int, max_len: int):
    """Returns (status_or_hit, tokens, score)."""
    buf = (C.c_int32 * max(1, max_len))()
    n = C.c_int32(0)
    sc = C.c_float(0.0)
    st = lib.card_cache_query(handle, verified_token, max_len, buf, C.byref(n), C.byref(sc))
    return st, list(buf[: n.value]), sc.value


def card_cache_correct(handle, verified_tokens) -> int:
    return lib.card_cache_correct(handle, _i32(verified_tokens), len(verified_tokens))


def card_cache_epoch(handle) -> int:
    return lib.card_cache_epoch(handle)


def card_cache_depth(handle) -> int:
    return lib.card_cache_depth(handle)


def card_cache_read_level(handle, level: int, K: int):
    t = (C.c_int32 * K)()
    p = (C.c_int32 * K)()
    s = (C.c_float * K)()
    n = lib.card_cache_read_level(handle, level, t, p, s)
    if n < 0:
        return n, [], [], []
    return n, list(t[:n]), list(p[:n]), list(s[:n])
