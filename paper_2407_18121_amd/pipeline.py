"""Buffers and call order of the hot path for one layer (marshalling only; all compute is in the library).

prefill():  ec_prefill_score -> ec_select_anchors -> ec_merge_compact      (Sec. 3.3 Instruction Encoding)
decode():   ec_evict_index (host) -> ec_decode_step                        (Sec. 3.3 Output Generation)
extend():   ec_chunk_score -> ec_select_anchors -> ec_remerge_compact      (a later turn: chat history is
                                                                            compressed again with the new chunk)
"""
from __future__ import annotations

import torch

from . import binding as ec


class LayerState:
    """Device buffers of one layer's compressed cache plus the bookkeeping integers of Alg. 1."""

    def __init__(self, B, H, D, T, n_anchor, cap, dtype: torch.dtype, gamma, G=1, recent=25,
                 protect_first=1, protect_last=1, device="cuda", keep_assign=False):
        self.B, self.H, self.D, self.T, self.G = B, H, D, T, G
        self.n_anchor, self.cap, self.gamma, self.recent = n_anchor, cap, gamma, recent
        self.protect_first, self.protect_last = protect_first, protect_last
        self.k_cache = torch.zeros((B, H, cap, D), dtype=dtype, device=device)
        self.v_cache = torch.zeros((B, H, cap, D), dtype=dtype, device=device)
        self.pos = torch.zeros((B, G, cap), dtype=torch.int32, device=device)
        self.score = torch.empty((B, G, T), dtype=torch.float32, device=device)
        self.anchor_idx = torch.empty((B, G, n_anchor), dtype=torch.int32, device=device)
        self.counts = torch.empty((B, G, n_anchor), dtype=torch.int32, device=device)
        self.assign = torch.empty((B, G, T), dtype=torch.int32, device=device) if keep_assign else None
        self.cache_len = 0
        self.n_seen = 0

    def prefill(self, q, k, v, scale, ws_prefill, out=None, lse=None):
        ec.ec_prefill_score(q, k, v, out, lse, self.score, scale, ws_prefill)
        ec.ec_select_anchors(self.score, self.n_anchor, self.protect_first, self.protect_last, self.anchor_idx)
        ec.ec_merge_compact(k, v, self.anchor_idx, self.k_cache, self.v_cache, self.counts, self.assign, self.pos)
        self.cache_len = self.n_anchor
        self.n_seen = self.T

    def decode(self, q, k_new, v_new, scale, out, ws_decode):
        self.n_seen += 1
        idx = ec.ec_evict_index(self.n_seen, self.cache_len + 1, self.gamma[0], self.gamma[1],
                                recent=self.recent, protect_first=self.protect_first)
        ec.ec_decode_step(q, k_new, v_new, self.k_cache, self.v_cache, self.pos, self.cache_len, idx,
                          self.n_seen - 1, scale, out, ws_decode)
        if idx < 0:
            self.cache_len += 1
        return idx

    def extend(self, q, k, v, scale, ws_chunk, out=None, lse=None):
        """A later multi-token pass: the chunk's K/V rows go behind the cache rows, the chunk's queries score
        every row of [cache | chunk], and the rows are merged again (Alg. 1's plain mean) into
        ceil(gamma * tokens seen) rows."""
        T_new = q.shape[2]
        P, L = self.cache_len, self.cache_len + T_new
        if L > self.cap:
            raise ValueError(f"cache capacity {self.cap} cannot hold {P} rows + a chunk of {T_new}")
        self.k_cache[:, :, P:L].copy_(k)
        self.v_cache[:, :, P:L].copy_(v)
        self.pos[:, :, P:L] = torch.arange(self.n_seen, self.n_seen + T_new, dtype=torch.int32, device=self.pos.device)
        self.n_seen += T_new
        n_new = -(-self.gamma[0] * self.n_seen // self.gamma[1])
        n_new = max(min(n_new, L), self.protect_first + self.protect_last)
        dev = self.k_cache.device
        self.score = torch.empty((self.B, self.G, L), dtype=torch.float32, device=dev)
        ec.ec_chunk_score(q, self.k_cache, self.v_cache, P, out, lse, self.score, scale, ws_chunk)
        self.anchor_idx = torch.empty((self.B, self.G, n_new), dtype=torch.int32, device=dev)
        ec.ec_select_anchors(self.score, n_new, self.protect_first, self.protect_last, self.anchor_idx)
        src_pos = self.pos[:, :, :L].clone()  # the merge writes self.pos while it reads the old map
        k_next, v_next = torch.zeros_like(self.k_cache), torch.zeros_like(self.v_cache)
        self.counts = torch.empty((self.B, self.G, n_new), dtype=torch.int32, device=dev)
        ec.ec_remerge_compact(self.k_cache, self.v_cache, L, self.anchor_idx, k_next, v_next, src_pos=src_pos,
                              counts=self.counts, pos=self.pos)
        self.k_cache, self.v_cache = k_next, v_next
        self.n_anchor = self.cache_len = n_new
        return n_new
