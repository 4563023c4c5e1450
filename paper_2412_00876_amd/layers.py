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


class DecoderStack:
    """Prefill through a stack of LLaMA-family decoder layers (RMSNorm, rotary attention, SwiGLU feed-forward; the
    decoder the paper sparsifies) with the one-time token reduction after layer l.  Sequencing only.

    weights: list of dicts per layer with device tensors Wq, Wk, Wv [H*Dh, d], Wo [d, H*Dh], Wg, Wu [d_ff, d],
    Wd [d, d_ff] (bfloat16) and g1, g2 [d] (float32).  One paged cache per layer receives that layer's K/V:
    all tokens for layers before l, the kept tokens after.
    """

    RMS_EPS = 1e-5
    ROPE_BASE = 10000.0

    def __init__(self, weights, l: int, B: int, H: int, Dh: int, d: int, d_ff: int, sumN: int, vision_rows: int,
                 max_seq_len: Optional[int] = None, extra_tokens: int = 0, device="cuda:0"):
        self.W, self.l, self.B, self.H, self.Dh, self.d, self.d_ff, self.sumN = weights, l, B, H, Dh, d, d_ff, sumN
        self.logits = torch.zeros((max(1, vision_rows), 2), dtype=torch.float32, device=device)
        self.dummy_logits = torch.zeros((max(1, sumN), 2), dtype=torch.float32, device=device)
        self.mask_all = torch.zeros(sumN, dtype=torch.uint8, device=device)
        bf = torch.bfloat16
        z = lambda *shape: torch.zeros(shape, dtype=bf, device=device)
        self.X, self.X2, self.Hn = z(sumN, d), z(sumN, d), z(sumN, d)
        self.Q, self.A = z(sumN, H, Dh), z(sumN, H, Dh)
        self.G, self.F = z(sumN, d_ff), z(sumN, d_ff)
        self.err = torch.zeros(1, dtype=torch.int32, device=device)
        self.caches = []
        for _ in weights:
            mp = ((max_seq_len or sumN) + extra_tokens + P.PAGE_SIZE - 1) // P.PAGE_SIZE   # pages per sequence
            pages = torch.zeros((B * mp, 2, H, P.PAGE_SIZE, Dh), dtype=bf, device=device)
            bt = torch.arange(B * mp, dtype=torch.int32, device=device).reshape(B, mp).contiguous()
            self.caches.append(P.KVCache(pages, bt, torch.zeros(B, dtype=torch.int32, device=device)))
        self.ws_select = torch.zeros(P.dllava_select_compact_workspace(B, sumN), dtype=torch.uint8, device=device)
        self.keep_mask = torch.zeros(sumN, dtype=torch.uint8, device=device)
        self.kept_idx = torch.zeros(sumN, dtype=torch.int32, device=device)
        self.out_off = torch.zeros(B + 1, dtype=torch.int32, device=device)
        self.full_idx = torch.zeros(sumN, dtype=torch.int32, device=device)
        self.full_off = torch.zeros(B + 1, dtype=torch.int32, device=device)
        # decode: one row per sequence
        self.xd, self.hd = z(B, d), z(B, d)
        self.qd, self.kd, self.vd, self.od = z(B, H, Dh), z(B, H, Dh), z(B, H, Dh), z(B, H, Dh)
        self.fd = z(B, d_ff)
        self.ones = torch.ones(B, dtype=torch.uint8, device=device)
        self.logits_d = torch.zeros((B, 2), dtype=torch.float32, device=device)
        self.keep_d = torch.zeros(B, dtype=torch.uint8, device=device)
        zb = lambda n: torch.zeros(n, dtype=torch.uint8, device=device)
        self.ws_few = zb(max(P.dllava_decode_proj_workspace(3 * H * Dh, d), P.dllava_decode_proj_workspace(2 * d_ff, d),
                             P.dllava_linear_few_workspace(d, H * Dh), P.dllava_linear_few_workspace(d, d_ff)))
        self.ws_decode = zb(P.dllava_decode_workspace(B, H, Dh, self.caches[0].max_pages_per_seq))

    def decode_step(self, x_new, pos, theta: float, predictor):
        """One generated token per sequence through all layers.  x_new [B, d]; pos [B] int32: the token's position in the
        ORIGINAL sequence; predictor(X, logits): the output-text predictor on the B hidden rows after layer l.  Layers
        before l append the token to their caches; later layers append it where the shared decision says keep.
        Returns the output rows [B, d] (a view) — the decision is left in self.keep_d / self.logits_d."""
        W_, d, ff, H, Dh, B, BF = self.W, self.d, self.d_ff, self.H, self.Dh, self.B, P.BF16
        few = lambda x, K, Wm, N, act, res, y: P.dllava_linear_few(x, K, B, K, Wm, None, N, act, res, y, N, BF, self.ws_few)
        self.xd.copy_(x_new)
        X = self.xd
        for i, Wl in enumerate(W_):
            if i == self.l:
                predictor(X, self.logits_d)
            P.dllava_rms_norm(X, d, B, d, Wl["g1"], self.RMS_EPS, self.hd, d, BF)
            P.dllava_qkv_few(self.hd, d, B, d, Wl["Wq"], Wl["Wk"], Wl["Wv"], H, Dh, pos, self.ROPE_BASE, self.qd, self.kd,
                             self.vd, BF, self.ws_few)
            if i < self.l:
                P.dllava_decode_attn_append(self.qd, self.kd, self.vd, B, None, 0.0, self.ones, self.caches[i], Dh ** -0.5,
                                            self.od, None, self.err, self.ws_decode)
            else:
                P.dllava_decode_attn_append(self.qd, self.kd, self.vd, B, self.logits_d, theta, None, self.caches[i],
                                            Dh ** -0.5, self.od, self.keep_d, self.err, self.ws_decode)
            few(self.od, H * Dh, Wl["Wo"], d, 0, X, X)
            P.dllava_rms_norm(X, d, B, d, Wl["g2"], self.RMS_EPS, self.hd, d, BF)
            P.dllava_gated_few(self.hd, d, B, d, Wl["Wg"], Wl["Wu"], ff, self.fd, ff, BF, self.ws_few)
            few(self.fd, ff, Wl["Wd"], d, 0, X, X)
        return X

    def kv_bytes(self) -> int:
        """Bytes of K and V held by all layers right now."""
        return int(sum(int(c.cache_len.sum().item()) for c in self.caches)) * 2 * self.H * self.Dh * 2

    def _layer(self, i: int, X, rows: int, off, pos):
        """One decoder layer in place on the first `rows` rows of X (rows = host count of off[B])."""
        W, d, ff, H, Dh, BF = self.W[i], self.d, self.d_ff, self.H, self.Dh, P.BF16
        c = self.caches[i]
        P.dllava_rms_norm(X, d, rows, d, W["g1"], self.RMS_EPS, self.Hn, d, BF)
        P.dllava_qkv_project(self.Hn, d, rows, d, self.B, off, pos, W["Wq"], W["Wk"], W["Wv"], self.ROPE_BASE, self.Q, c,
                             self.err, BF)
        P.dllava_prefill_attn(self.Q, None, None, c, self.B, off, rows, H, Dh, Dh ** -0.5, self.A, BF)
        P.dllava_linear(self.A, H * Dh, rows, H * Dh, W["Wo"], None, d, 0, X, X, d, BF)
        P.dllava_rms_norm(X, d, rows, d, W["g2"], self.RMS_EPS, self.Hn, d, BF)
        P.dllava_linear(self.Hn, d, rows, d, W["Wg"], None, ff, 0, None, self.G, ff, BF)
        P.dllava_linear(self.Hn, d, rows, d, W["Wu"], None, ff, 2, self.G, self.F, ff, BF)
        P.dllava_linear(self.F, ff, rows, ff, W["Wd"], None, d, 0, X, X, d, BF)

    def prefill(self, x0, seq_off, vis_start, vis_len, keep_ratio: float, kept_rows: int, predictor):
        """x0 [sumN, d]: the decoder's input rows.  predictor(X, logits): fills logits [sum vis_len, 2] from the rows of
        X's vision spans (a call of dllava_score or dllava_predict).  kept_rows: host count of the rows that stay,
        sum over sequences of text rows + floor(keep_ratio * vision rows).  Returns the final rows (a view)."""
        self.X.copy_(x0)
        # positions of all tokens: the "everything kept" decisions
        P.dllava_select_compact(self.dummy_logits, self.B, seq_off, vis_start, vis_len, self.sumN, P.MODE_TOPK, 1.0, 0.0, None, None, 0,
                                None, None, None, None, None, self.mask_all, self.full_idx, self.full_off, self.err,
                                P.BF16, self.ws_select)
        X, rows, off, pos = self.X, self.sumN, self.full_off, self.full_idx
        for i in range(len(self.W)):
            if i == self.l:
                predictor(X, self.logits)
                P.dllava_select_compact(self.logits, self.B, seq_off, vis_start, vis_len, self.sumN, P.MODE_TOPK, keep_ratio,
                                        0.0, X, self.X2, self.d, None, None, None, None, None, self.keep_mask, self.kept_idx,
                                        self.out_off, self.err, P.BF16, self.ws_select)
                X, rows, off, pos = self.X2, kept_rows, self.out_off, self.kept_idx
            self._layer(i, X, rows, off, pos)
        return X[:rows]
