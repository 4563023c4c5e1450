"""Attention state of a stack of decoder layers under the paper's one-time decision (Sec. 3.3: the predictors run
once, after decoder layer l, and their decisions are shared by all subsequent layers; l = 2 in the paper).

Sequencing only: every step is a call into the library.  Layers 1..l keep FULL caches (every prompt token, every
generated token); layers l+1..L keep the reduced prompt and the generated tokens whose shared decision is "keep".
The per-layer tensors (hidden states, Q, K, V) are the caller's: the rest of a decoder layer is outside this library.
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import binding as P


class SparsifiedLayers:
    def __init__(self, n_layers: int, l: int, B: int, H: int, Dh: int, full_capacity: int, reduced_capacity: int,
                 dtype: torch.dtype, device="cuda:0"):
        assert 0 <= l <= n_layers
        self.L, self.l, self.B, self.H, self.Dh = n_layers, l, B, H, Dh
        self.code = P.dtype_code(dtype)
        self.es = 2 if dtype == torch.bfloat16 else 4
        self.caches: List[P.KVCache] = []
        for layer in range(n_layers):
            cap = full_capacity if layer < l else reduced_capacity
            mp = (cap + P.PAGE_SIZE - 1) // P.PAGE_SIZE
            pages = torch.zeros((B * mp, 2, H, P.PAGE_SIZE, Dh), dtype=dtype, device=device)
            bt = torch.arange(B * mp, dtype=torch.int32, device=device).reshape(B, mp).contiguous()
            self.caches.append(P.KVCache(pages, bt, torch.zeros(B, dtype=torch.int32, device=device)))
        self.err = torch.zeros(1, dtype=torch.int32, device=device)
        self.ones = torch.ones(B, dtype=torch.uint8, device=device)
        self.scale = Dh ** -0.5
        self.ws_decode = torch.zeros(max(P.dllava_decode_workspace(B, H, Dh, c.max_pages_per_seq) for c in self.caches),
                                     dtype=torch.uint8, device=device)
        self.kept_idx = self.out_off = self.full_idx = None
        self.seq_off = None

    # ---- prefill ---------------------------------------------------------------------------------------------
    def begin(self, seq_off, vis_start, vis_len, sumN: int):
        """Token layout of the batch; also prepares the "everything kept" decisions of layers 1..l."""
        dev = seq_off.device
        self.seq_off, self.vis_start, self.vis_len, self.sumN = seq_off, vis_start, vis_len, sumN
        self.ws_select = torch.zeros(P.dllava_select_compact_workspace(self.B, sumN), dtype=torch.uint8, device=dev)
        self.full_idx = torch.zeros(sumN, dtype=torch.int32, device=dev)
        self.full_off = torch.zeros(self.B + 1, dtype=torch.int32, device=dev)
        mask = torch.zeros(sumN, dtype=torch.uint8, device=dev)
        no_logits = torch.zeros((max(1, sumN), 2), dtype=torch.float32, device=dev)
        P.dllava_select_compact(no_logits, self.B, seq_off, vis_start, vis_len, sumN, P.MODE_TOPK, 1.0, 0.0, None, None, 0,
                                None, None, None, None, None, mask, self.full_idx, self.full_off, self.err, self.code,
                                self.ws_select)

    def prefill_layer(self, layer: int, Q, K, V, O, Q_scratch):
        """Attention of one layer over its token set, K/V into the layer's cache.  Q, K, V: [sumN, H, Dh] of ALL tokens."""
        kept, off = (self.full_idx, self.full_off) if layer < self.l else (self.kept_idx, self.out_off)
        assert kept is not None, "decide() comes before the first layer beyond l"
        c = self.caches[layer]
        P.dllava_compact(self.B, self.seq_off, kept, off, self.sumN, None, None, 0, Q, Q_scratch, K, V, c, self.err, self.code)
        P.dllava_prefill_attn(Q_scratch, None, None, c, self.B, off, self.sumN, self.H, self.Dh, self.scale, O, self.code)

    def decide(self, logits, keep_ratio: float, hidden=None, hidden_out=None, d: int = 0):
        """The one-time decision after layer l, from the image predictor's logits; optionally compacts the hidden states."""
        dev = logits.device
        self.keep_mask = torch.zeros(self.sumN, dtype=torch.uint8, device=dev)
        self.kept_idx = torch.zeros(self.sumN, dtype=torch.int32, device=dev)
        self.out_off = torch.zeros(self.B + 1, dtype=torch.int32, device=dev)
        P.dllava_select_compact(logits, self.B, self.seq_off, self.vis_start, self.vis_len, self.sumN, P.MODE_TOPK,
                                keep_ratio, 0.0, hidden, hidden_out, d, None, None, None, None, None, self.keep_mask,
                                self.kept_idx, self.out_off, self.err, self.code, self.ws_select)

    # ---- decode ----------------------------------------------------------------------------------------------
    def decode_layer(self, layer: int, q, k, v, o, keep: Optional[torch.Tensor]):
        """One decode step of one layer.  keep [B] uint8: the shared decision of this token (layers beyond l)."""
        ov = self.ones if layer < self.l else keep
        P.dllava_decode_attn_append(q, k, v, self.B, None, 0.0, ov, self.caches[layer], self.scale, o, None, self.err,
                                    self.ws_decode)

    # ---- accounting ------------------------------------------------------------------------------------------
    def kv_bytes(self) -> int:
        """Bytes of K and V held by all layers right now."""
        per_token = 2 * self.H * self.Dh * self.es
        return int(sum(int(c.cache_len.sum().item()) for c in self.caches)) * per_token
