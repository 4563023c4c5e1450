"""CPU oracle for a stack of decoder layers with the paper's one-time token reduction (Sec. 3.1, Eq. 2-3: a decoder
layer is FFN(MHA(.)) with the projections W^Q, W^K, W^V, W^O; Sec. 3.3: the predictors run once, after layer l, and
all subsequent layers work on the reduced token set).

TEST INFRASTRUCTURE ONLY: imported by the tests and the benchmark's checks; the product path never imports it.

The paper sparsifies the LLaMA-family decoder of LLaVA-1.5 and does not restate that layer.  It is taken here in its
published form (parity unpinned against the paper, pinned against the reference implementation of that decoder in the
`transformers` package): pre-norm residual layer, RMSNorm (eps 1e-5, learned scale), rotary positions on q and k in the
half-split pairing, causal attention with scale 1/sqrt(Dh), no biases, SwiGLU feed-forward
    x <- x + W_O Attention(q, k, v),  [q|k|v] = W^{Q,K,V} RMSNorm(x)
    x <- x + W_down (SiLU(W_gate h) * (W_up h)),  h = RMSNorm(x).
After the reduction the kept tokens keep their ORIGINAL positions (as in dllava_ref.qkv_project).

Precision: tensors written between two operations (norm outputs, q/k/v, attention output, the residual stream after
each addition, the gate, the gated product) are rounded to the storage type when round_intermediates is set; sums are
float64.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np

from . import dllava_ref as R

RMS_EPS = 1e-5
ROPE_BASE = 10000.0


def rms_norm(x: np.ndarray, w, eps: float = RMS_EPS) -> np.ndarray:
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * np.asarray(w, np.float64)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def _st(a, dtype, on):
    return R.widen(R.narrow(a, dtype), dtype) if on else a


def decoder_layer(x: np.ndarray, off, pos, L: Dict, H: int, Dh: int, dtype: str, round_intermediates: bool = True,
                  cache: Optional[R.PagedCache] = None) -> np.ndarray:
    """One layer over the rows x [M, d] (float64 values; representable in dtype when rounding is on).

    off [B+1]: sequences; pos [M]: position of every row in its ORIGINAL sequence.  K/V go to `cache` when given.
    """
    rnd = round_intermediates
    M = x.shape[0]
    h1 = _st(rms_norm(x, L["g1"]), dtype, rnd)
    q, k, v = (h1 @ R.widen(L[n], dtype).T for n in ("Wq", "Wk", "Wv"))
    q = _st(R.rope_rotate(q.reshape(M, H, Dh), pos, ROPE_BASE), dtype, rnd)
    k = _st(R.rope_rotate(k.reshape(M, H, Dh), pos, ROPE_BASE), dtype, rnd)
    v = _st(v.reshape(M, H, Dh), dtype, rnd)
    if cache is not None:
        ks, vs = R.narrow(k, dtype), R.narrow(v, dtype)
        for b in range(len(off) - 1):
            for t in range(int(off[b + 1] - off[b])):
                cache.put(b, t, ks[off[b] + t], vs[off[b] + t])
            cache.cache_len[b] = int(off[b + 1] - off[b])
    a = np.zeros((M, H, Dh))
    scale = 1.0 / math.sqrt(Dh)
    for b in range(len(off) - 1):
        r0, r1 = int(off[b]), int(off[b + 1])
        n = r1 - r0
        if n == 0:
            continue
        causal = np.tril(np.ones((n, n), dtype=bool))
        for h in range(H):
            s = np.where(causal, (q[r0:r1, h] @ k[r0:r1, h].T) * scale, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            a[r0:r1, h] = (e @ v[r0:r1, h]) / e.sum(axis=1, keepdims=True)
    a = _st(a.reshape(M, H * Dh), dtype, rnd)
    x = _st(x + a @ R.widen(L["Wo"], dtype).T, dtype, rnd)
    h2 = _st(rms_norm(x, L["g2"]), dtype, rnd)
    gate = _st(h2 @ R.widen(L["Wg"], dtype).T, dtype, rnd)
    f = _st(silu(gate) * (h2 @ R.widen(L["Wu"], dtype).T), dtype, rnd)
    return _st(x + f @ R.widen(L["Wd"], dtype).T, dtype, rnd)


def decoder_prefill(x0, seq_off, vis_start, vis_len, layers: List[Dict], l: int, keep_ratio: float, predictor, H: int,
                    Dh: int, dtype: str, round_intermediates: bool = True, caches: Optional[list] = None):
    """Prefill through all layers; after layer l (1-based count of full layers) the image predictor's logits decide
    which image tokens stay (Eq. 11) and the later layers see the reduced set only.

    predictor(x_rows_stored) -> logits [rows, 2] for the rows of the vision spans (in span order).
    Returns (x_final [rows*, d] float64, kept_idx, out_off, logits): for l >= len(layers) nothing is reduced
    (kept_idx = every position).
    """
    seq_off = np.asarray(seq_off)
    B = len(seq_off) - 1
    x = R.widen(x0, dtype)
    off = seq_off.copy()
    pos = np.concatenate([np.arange(seq_off[b + 1] - seq_off[b]) for b in range(B)]).astype(np.int64)
    idx, logits = pos.copy(), None
    for i, L in enumerate(layers):
        if i == l:
            vis = np.concatenate([np.arange(seq_off[b] + vis_start[b], seq_off[b] + vis_start[b] + vis_len[b])
                                  for b in range(B)]).astype(np.int64)
            logits = predictor(R.narrow(x[vis], dtype))
            _, idx, off = R.select(logits, seq_off, vis_start, vis_len, R.TOPK, keep_ratio, 0.0)
            src = np.concatenate([seq_off[b] + idx[off[b]:off[b + 1]] for b in range(B)]).astype(np.int64)
            x, pos = x[src], idx[: off[-1]].astype(np.int64)
        x = decoder_layer(x, off, pos, L, H, Dh, dtype, round_intermediates, cache=caches[i] if caches else None)
    return x, idx, off, logits


def decoder_decode_step(x_new, pos, layers: List[Dict], caches: list, l: int, theta: float, predictor, H: int, Dh: int,
                        dtype: str, round_intermediates: bool = True, keep_override=None):
    """One generated token per sequence through all layers (Eq. 3 per layer; Eq. 6 for the caches).

    x_new [B, d] stored: the token's input rows; pos [B]: its position in the ORIGINAL sequence (dropped tokens count).
    Layers before l append the token's K/V to their caches unconditionally; after layer l the output-text
    predictor's logits on the hidden rows decide once (margin > theta), and every later layer appends only if kept
    (the token still takes part in its own attention in every layer).  Returns (x_out [B, d] float64, keep, logits).
    """
    rnd = round_intermediates
    x = R.widen(x_new, dtype)
    B = x.shape[0]
    scale = 1.0 / math.sqrt(Dh)
    keep, logits = np.ones(B, np.uint8), None
    for i, L in enumerate(layers):
        if i == l:
            logits = predictor(R.narrow(x, dtype))
            keep = np.asarray(keep_override, np.uint8) if keep_override is not None else R.decode_keep(logits, theta)
        h1 = _st(rms_norm(x, L["g1"]), dtype, rnd)
        q, k, v = (h1 @ R.widen(L[n], dtype).T for n in ("Wq", "Wk", "Wv"))
        q = R.rope_rotate(q.reshape(B, H, Dh), pos, ROPE_BASE)
        k = R.rope_rotate(k.reshape(B, H, Dh), pos, ROPE_BASE)
        o, err = R.decode_attn_append(R.narrow(q, dtype), R.narrow(k, dtype), R.narrow(v.reshape(B, H, Dh), dtype),
                                      keep if i >= l else np.ones(B, np.uint8), caches[i], scale)
        if np.any(err):
            raise ValueError("cache capacity exceeded")
        a = _st(o.reshape(B, H * Dh), dtype, rnd)
        x = _st(x + a @ R.widen(L["Wo"], dtype).T, dtype, rnd)
        h2 = _st(rms_norm(x, L["g2"]), dtype, rnd)
        gate = _st(h2 @ R.widen(L["Wg"], dtype).T, dtype, rnd)
        f = _st(silu(gate) * (h2 @ R.widen(L["Wu"], dtype).T), dtype, rnd)
        x = _st(x + f @ R.widen(L["Wd"], dtype).T, dtype, rnd)
    return x, keep, logits
