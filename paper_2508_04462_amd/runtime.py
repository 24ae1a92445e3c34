"""Device-buffer plumbing around the C ABI: torch allocates, libcard computes."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import binding as B


def make_cfg(shape, max_ctx: int, max_r: int = 32, grid_wgs: int = 0) -> B.CardModelCfg:
    """shape: any object with the ModelShape fields."""
    max_ctx = (max_ctx + 15) // 16 * 16
    return B.CardModelCfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                          shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps, 16, max_ctx, max_r, grid_wgs)


_LANE_STREAMS: Dict[str, list] = {}


def _lane_streams(device, lanes: int) -> list:
    """Streams for kernels that are to run side by side, created once per device and shared by
    everything that needs such streams: a process has few hardware queues (four by default) and
    streams are mapped onto them in turn, so every further stream risks sharing a queue with
    another one, and two kernels on one queue run one after the other."""
    have = _LANE_STREAMS.setdefault(str(device), [])
    while len(have) < lanes:
        have.append(torch.cuda.Stream(device=device))
    return have[:lanes]


def _check(st: int, where: str) -> None:
    if st != B.CARD_OK:
        raise B.CardError(st, where)


class Target:
    """The target model's device state: packed weights, workspace, paged KV cache."""

    def __init__(self, shape, max_ctx: int, max_r: int = 32, device: str = "cuda:0",
                 page_order: Optional[Sequence[int]] = None, grid_wgs: int = 0, pool_fill: Optional[int] = None):
        """pool_fill: byte value the KV page pools start with (tests; None = whatever torch.empty
        hands out)."""
        if not torch.cuda.is_available():
            raise RuntimeError("libcard needs a GPU: there is no CPU path")
        self.device = torch.device(device)
        self.cfg = make_cfg(shape, max_ctx, max_r, grid_wgs)
        wbytes = B.card_packed_weight_bytes(self.cfg)
        if wbytes == 0:
            raise B.CardError(B.CARD_EINVAL, "card_packed_weight_bytes")
        self.packed = torch.empty(wbytes, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(B.card_workspace_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        _check(B.card_workspace_init(self.cfg, self.workspace, self._stream()), "card_workspace_init")
        self.n_pages = self.cfg.max_ctx // 16
        pool = B.card_kv_pool_bytes(self.cfg, self.n_pages)
        self.k_pages = torch.empty(pool, dtype=torch.uint8, device=self.device)
        self.v_pages = torch.empty(pool, dtype=torch.uint8, device=self.device)
        if pool_fill is not None:
            self.k_pages.fill_(pool_fill)
            self.v_pages.fill_(pool_fill)
        order = list(range(self.n_pages)) if page_order is None else [int(p) for p in page_order]
        assert sorted(order) == list(range(self.n_pages))
        self.block_table = torch.tensor(order, dtype=torch.int32, device=self.device)
        self.out = torch.zeros(4, dtype=torch.int32, device=self.device)
        self.row_argmax = torch.zeros(32, dtype=torch.int32, device=self.device)
        self.cand = torch.zeros(32, dtype=torch.int32, device=self.device)

    # -- weights
    def pack(self, name: str, layer: int, src: torch.Tensor) -> None:
        src = src.to(self.device).contiguous()
        st = B.card_weights_pack_tensor(self.cfg, B.TENSOR_IDS[name], layer, src, self.packed, self._stream())
        _check(st, f"card_weights_pack_tensor({name}, {layer})")
        torch.cuda.current_stream(self.device).synchronize()  # src may be freed by the caller

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def kv(self, pending: int) -> B.CardKV:
        return B.CardKV(self.k_pages.data_ptr(), self.v_pages.data_ptr(), self.block_table.data_ptr(),
                        self.n_pages, int(pending))

    # -- one verification step
    def enqueue_verify(self, ctx_len: int, pending: int, r: int, logits: Optional[torch.Tensor] = None,
                       cand: Optional[torch.Tensor] = None, sampling: Optional[B.CardSampling] = None) -> int:
        """Enqueue on the current stream; candidates come from `cand` (device int32) or from
        self.cand[:r].  No synchronisation."""
        kv = self.kv(pending)
        cand = self.cand if cand is None else cand
        if sampling is not None:
            return B.card_verify_sampled(self.cfg, self.packed, kv, ctx_len, cand, r, sampling, self.workspace,
                                         self._stream(), self.out, self.row_argmax, logits)
        if logits is None:
            return B.card_verify(self.cfg, self.packed, kv, ctx_len, cand, r, self.workspace,
                                 self._stream(), self.out, self.row_argmax)
        return B.card_verify_debug_logits(self.cfg, self.packed, kv, ctx_len, cand, r, self.workspace,
                                          self._stream(), self.out, self.row_argmax, logits)

    def verify(self, ctx_len: int, pending: int, cand: Sequence[int], want_logits: bool = False,
               temperature: float = 0.0, seed: int = 0) -> Dict:
        r = len(cand)
        if 0 < r <= 32:
            self.cand[:r] = torch.tensor([int(c) for c in cand], dtype=torch.int32, device=self.device)
        logits = None
        if want_logits:
            logits = torch.empty((max(r, 1), self.cfg.vocab), dtype=torch.float32, device=self.device)
        sampling = B.CardSampling(float(temperature), int(seed)) if temperature > 0 else None
        _check(self.enqueue_verify(ctx_len, pending, r, logits, sampling=sampling), "card_verify")
        torch.cuda.current_stream(self.device).synchronize()
        o = self.out.tolist()
        res = {"accepted_len": o[0], "correction_token": o[1], "kv_first_slot": o[2], "kv_count": o[3],
               "row_argmax": self.row_argmax[:r].tolist()}
        if want_logits:
            res["logits"] = logits.cpu()
        return res

    # -- draft side: one level of cache construction
    def draft_level(self, ctx_len: int, tokens: Sequence[int], positions: Sequence[int], first_slot: int,
                    mask_rows: Sequence[Sequence[int]], mask_base: int, k: int, want_logits: bool = False) -> Dict:
        """Forward the tree nodes `tokens` (at most max_r of them) with card_draft_level; returns the
        device tensors topk_tokens [n][k] (int32), topk_probs [n][k] (fp32) and, on request, the logits."""
        n, words = len(tokens), len(mask_rows[0])
        dev = self.device
        tok = torch.tensor([int(t) for t in tokens], dtype=torch.int32, device=dev)
        pos = torch.tensor([int(p) for p in positions], dtype=torch.int32, device=dev)
        mask = torch.tensor([[int(w) - (1 << 32) if int(w) >= (1 << 31) else int(w) for w in row] for row in mask_rows],
                            dtype=torch.int32, device=dev)
        rows = B.CardTreeRows(tok.data_ptr(), pos.data_ptr(), int(first_slot), mask.data_ptr(), words, int(mask_base))
        tk = torch.full((n, k), -7, dtype=torch.int32, device=dev)
        tp = torch.zeros((n, k), dtype=torch.float32, device=dev)
        logits = torch.empty((n, self.cfg.vocab), dtype=torch.float32, device=dev) if want_logits else None
        _check(B.card_draft_level(self.cfg, self.packed, self.kv(-1), ctx_len, rows, n, k, self.workspace, self._stream(),
                                  tk, tp, logits), "card_draft_level")
        torch.cuda.current_stream(dev).synchronize()
        res = {"topk_tokens": tk, "topk_probs": tp}
        if want_logits:
            res["logits"] = logits.cpu()
        return res

    # -- a level wider than one call: several calls side by side
    def enable_lanes(self, lanes: int) -> None:
        """Prepare `lanes` workspaces and streams for draft_level_wide.  The model must have been
        created with grid_wgs set so that lanes * grid_wgs workgroups fit the GPU: every call of a
        level then runs on its own share of the compute units."""
        cus = torch.cuda.get_device_properties(self.device).multi_processor_count
        if self.cfg.grid_wgs <= 0 or lanes * self.cfg.grid_wgs > cus:
            raise ValueError("lanes * grid_wgs must fit the compute units")
        self._lane_ws = [self.workspace]
        for _ in range(lanes - 1):
            ws = torch.empty_like(self.workspace)
            _check(B.card_workspace_init(self.cfg, ws, self._stream()), "card_workspace_init")
            self._lane_ws.append(ws)
        self._lane_streams = _lane_streams(self.device, lanes)
        torch.cuda.current_stream(self.device).synchronize()

    def draft_level_wide(self, ctx_len: int, tokens: Sequence[int], positions: Sequence[int], first_slot: int,
                         mask_rows: Sequence[Sequence[int]], mask_base: int, k: int) -> Dict:
        """card_draft_level for a level of any width: the rows are cut into calls of at most 32, `lanes`
        of them at a time enqueued side by side, each on its own stream with its own workspace
        (peers of a level never see each other, so the calls are independent; they share the weights
        and the KV cache and write different slots; a lane's calls follow each other on its stream).
        Same results as the calls one after the other."""
        n, words, dev = len(tokens), len(mask_rows[0]), self.device
        lanes = len(self._lane_ws)
        tok = torch.tensor([int(t) for t in tokens], dtype=torch.int32, device=dev)
        pos = torch.tensor([int(p) for p in positions], dtype=torch.int32, device=dev)
        mask = torch.tensor([[int(w) - (1 << 32) if int(w) >= (1 << 31) else int(w) for w in row] for row in mask_rows],
                            dtype=torch.int32, device=dev)
        tk = torch.full((n, k), -7, dtype=torch.int32, device=dev)
        tp = torch.zeros((n, k), dtype=torch.float32, device=dev)
        cur = torch.cuda.current_stream(dev)
        ready = torch.cuda.Event()
        ready.record(cur)
        calls = (n + 31) // 32
        calls = (calls + lanes - 1) // lanes * lanes  # full rounds of side-by-side calls, rows spread evenly
        per = min(32, ((n + calls - 1) // calls + 7) // 8 * 8)  # whole 8-row groups per call where the level allows
        done = []
        for i, c0 in enumerate(range(0, n, per)):
            c1 = min(n, c0 + per)
            lane = i % lanes
            st = self._lane_streams[lane]
            if i < lanes:
                st.wait_event(ready)
            rows = B.CardTreeRows(tok[c0:c1].data_ptr(), pos[c0:c1].data_ptr(), int(first_slot) + c0, mask[c0:c1].data_ptr(),
                                  words, int(mask_base))
            _check(B.card_draft_level(self.cfg, self.packed, self.kv(-1), ctx_len, rows, c1 - c0, k, self._lane_ws[lane],
                                      st.cuda_stream, tk[c0:c1], tp[c0:c1], None), "card_draft_level")
            ev = torch.cuda.Event()
            ev.record(st)
            done.append(ev)
        for ev in done:
            cur.wait_event(ev)
        cur.synchronize()
        return {"topk_tokens": tk, "topk_probs": tp}

    def prefill(self, tokens: Sequence[int], chunk: int = 32) -> int:
        """Build KV[0:n) with verify calls that carry no pending token; returns the arg-max after
        the last context token (the pending prediction g0)."""
        chunk = min(chunk, self.cfg.max_r)
        last = None
        for s in range(0, len(tokens), chunk):
            last = self.verify(s, -1, tokens[s:s + chunk])
        return last["row_argmax"][-1]

    def kv_gather(self, layer: int, first: int, count: int):
        shp = (count, self.cfg.n_kv_heads, self.cfg.head_dim)
        k = torch.empty(shp, dtype=torch.float32, device=self.device)
        v = torch.empty(shp, dtype=torch.float32, device=self.device)
        _check(B.card_kv_gather(self.cfg, self.kv(-1), layer, first, count, k, v, self._stream()), "card_kv_gather")
        torch.cuda.current_stream(self.device).synchronize()
        return k.cpu(), v.cpu()


class CandidateCache:
    """RAII wrapper of the host-side shared candidate cache."""

    def __init__(self, K: int, max_depth: int):
        st, self.h = B.card_cache_create(K, max_depth)
        _check(st, "card_cache_create")
        self.K = K

    def __del__(self):
        h, self.h = getattr(self, "h", None), None
        destroy = getattr(B, "card_cache_destroy", None)  # module globals may be gone at interpreter exit
        if h and destroy is not None:
            destroy(h)

    def write(self, level: int, tokens, parents, scores, epoch: Optional[int] = None) -> int:
        return B.card_cache_write(self.h, self.epoch() if epoch is None else epoch, level, tokens, parents, scores)

    def query(self, token: int, max_len: int):
        st, toks, score = B.card_cache_query(self.h, token, max_len)
        if st < 0:
            raise B.CardError(st, "card_cache_query")
        return bool(st), toks, score

    def correct(self, tokens) -> bool:
        st = B.card_cache_correct(self.h, tokens)
        if st < 0:
            raise B.CardError(st, "card_cache_correct")
        return bool(st)

    def epoch(self) -> int:
        return B.card_cache_epoch(self.h)

    def depth(self) -> int:
        return B.card_cache_depth(self.h)

    def level(self, l: int):
        return B.card_cache_read_level(self.h, l, self.K)
