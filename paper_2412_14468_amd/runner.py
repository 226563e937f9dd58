"""Sequencing of the C-ABI calls for one decode layer-step, and device-side holders of a layer's
tensors.  No arithmetic of the method lives here: every step is a kernel behind the C ABI."""
from __future__ import annotations

import math
from typing import List, Optional

import torch

from .binding import Context, KvCache, Mlp


class LayerState:
    """Device tensors of one attention layer: KV cache, key-code store, mapping weights, the step's
    query and outputs.  Tensors are caller-owned; the library only reads/writes through pointers."""

    def __init__(self, q, k, v, seq_lens, max_seq_len: int, w_q: List[torch.Tensor],
                 w_kv: List[torch.Tensor], k_per_seq: Optional[torch.Tensor], k_max: int,
                 page_table: Optional[torch.Tensor] = None, k_new=None, v_new=None,
                 codes: Optional[torch.Tensor] = None, q_codes: Optional[torch.Tensor] = None):
        dev = q.device
        self.q, self.k, self.v, self.seq_lens = q, k, v, seq_lens
        self.B, self.Hq, self.d = int(q.shape[0]), int(q.shape[1]), int(q.shape[2])
        self.Hkv = int(k.shape[1])
        self.page_table = page_table
        self.k_new, self.v_new = k_new, v_new
        self.codes = codes if codes is not None else torch.zeros(tuple(k.shape[:3]), dtype=torch.int32, device=dev)
        self.cache = KvCache(k, v, self.codes, seq_lens, max_seq_len, page_table=page_table)
        self.phi_q = Mlp(w_q) if w_q is not None else None
        self.phi_kv = Mlp(w_kv) if w_kv is not None else None
        self.k_per_seq, self.k_max = k_per_seq, int(k_max)
        self.q_codes = q_codes if q_codes is not None else torch.zeros((self.B, self.Hq), dtype=torch.int32, device=dev)
        self.idx = torch.zeros((self.B, self.Hq, self.k_max), dtype=torch.int32, device=dev)
        self.count = torch.zeros((self.B, self.Hq), dtype=torch.int32, device=dev)
        self.threshold = torch.zeros((self.B, self.Hq), dtype=torch.uint8, device=dev)
        self.out = torch.zeros((self.B, self.Hq, self.d), dtype=torch.bfloat16, device=dev)
        self.dense_out = torch.zeros_like(self.out)
        self.scale = 1.0 / math.sqrt(self.d)
        self.n_sink = self.n_local = 0
        self.pitch = self.k_max                      # entries per row of idx

    def set_window(self, n_sink: int, n_local: int) -> None:
        """Always keep the first n_sink and the most recent n_local tokens; k counts the rest."""
        self.n_sink, self.n_local = int(n_sink), int(n_local)
        self.pitch = self.k_max + self.n_sink + self.n_local
        self.idx = torch.zeros((self.B, self.Hq, self.pitch), dtype=torch.int32, device=self.q.device)


def layer_from_tensors(t: dict) -> LayerState:
    """LayerState over a dict of device tensors as made by workloads.device_tensors."""
    uniform_k = bool((t["k_per_seq_host"] == t["k_per_seq_host"][0]).all())
    return LayerState(t["q"], t["k"], t["v"], t["seq_lens"], int(t["seq_lens_host"].max()), t["w_q"], t["w_kv"],
                      None if uniform_k else t["k_per_seq"], int(t["k_per_seq_host"].max()),
                      page_table=t["page_table"], k_new=t["k_new"], v_new=t["v_new"])


def build_key_codes(ctx: Context, s: LayerState) -> None:
    """Prefill-side: (re)build the whole key-code store from the cached keys."""
    ctx.hashattn_encode_keys(s.phi_kv, None, None, s.B, max(s.cache.max_seq_len, 1), s.cache)


def decode_step(ctx: Context, s: LayerState, append: bool = False, separate_calls: bool = False) -> None:
    """[append] -> encode query -> SCORE + TOPK -> GATHER-ATT on torch's current stream: one call of
    hashattn_decode_step, or (separate_calls, or a layer without a query mapping) the entry points of the steps
    one after the other."""
    if s.phi_q is not None and not separate_calls:
        ctx.hashattn_decode_step(s.phi_kv if append else None, s.k_new if append else None, s.v_new if append else None,
                                 s.phi_q, s.q, s.cache, s.B, s.k_per_seq, s.k_max, s.n_sink, s.n_local, s.scale,
                                 s.q_codes, s.idx, s.count, s.threshold, s.out)
        return
    if append:
        ctx.hashattn_encode_keys(s.phi_kv, s.k_new, s.v_new, s.B, 1, s.cache)
    if s.phi_q is not None:
        ctx.hashattn_encode_query(s.phi_q, s.q, s.B, s.q_codes)
    score_topk(ctx, s)
    gather_attend(ctx, s)


def score_topk(ctx: Context, s: LayerState) -> None:
    if s.n_sink or s.n_local:
        ctx.hashattn_score_topk_window(s.q_codes, s.cache, s.B, s.k_per_seq, s.k_max, s.n_sink, s.n_local,
                                       s.idx, s.count, s.threshold)
    else:
        ctx.hashattn_score_topk(s.q_codes, s.cache, s.B, s.k_per_seq, s.k_max, s.idx, s.count, s.threshold)


def gather_attend(ctx: Context, s: LayerState) -> None:
    ctx.hashattn_gather_attend(s.q, s.cache, s.idx, s.count, s.B, s.pitch, s.scale, s.out)


def dense_step(ctx: Context, s: LayerState) -> None:
    ctx.hashattn_dense_attend(s.q, s.cache, s.B, s.scale, s.dense_out)
