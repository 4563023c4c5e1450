"""CPU oracle for the predictors in the form the paper's appendix describes (Appendix A.4.1,
"Details of Predictor Architecture").

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's
``cpu_baseline`` leg; the product path never imports it and shares no code with it.

What the appendix fixes
  * both predictors start with one linear layer that reduces the decoder width d to 512;
  * the image predictor then applies two vision-transformer blocks, the output-text predictor none
    (its decision depends on the current token only);
  * both end in a three-layer MLP 512 -> 256 -> 128 -> 2.

What it leaves open (its figure is not part of the text) and how it is read here -- "parity unpinned"
for each of these readings, nothing in the paper can confirm them:
  * the reducing linear layer has a bias and no activation;
  * a block is the pre-norm block of the vision transformer the appendix cites:
        z <- z + Wo . MHA(LN1(z)),     z <- z + W2 . GELU(W1 . LN2(z)),
    8 heads of 64, fused q|k|v projection, softmax(q k^T / 8) v over ALL image tokens of the same
    sequence (no causal mask, no tokens of other sequences, no position term, no class token),
    MLP width 2048, LayerNorm eps 1e-6, exact (erf) GELU, biases everywhere;
  * the MLP head has GELU after its first two layers and none after the last; there is no final norm;
  * column 0 of the two outputs is "drop", column 1 "keep" (Eq. 5).

Precision: weights and activations are stored in the working type (bfloat16 for the GPU path).  Every
tensor that the computation writes to memory between two layers -- the reduced features, each
LayerNorm output, q/k/v, the attention output, the residual stream after each addition, each hidden
activation -- is rounded to that type (round_intermediates=True); all arithmetic between two such
points is float64.  The logits leave in float32.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np

from .dllava_ref import gelu, narrow, widen

WIDTH = 512        # Appendix A.4.1: both predictors reduce the input to 512
HEADS = 8
MLP_WIDTH = 2048
HEAD_WIDTHS = (256, 128, 2)   # Appendix A.4.1: 512 -> 256 -> 128 -> 2
LN_EPS = 1e-6


def _stored(a: np.ndarray, dtype: str, on: bool) -> np.ndarray:
    """float64 -> storage type -> float64 (what the next layer reads back)."""
    return widen(narrow(a, dtype), dtype) if on else a


def linear(x: np.ndarray, W, b, dtype: str) -> np.ndarray:
    """x W^T + b in float64; W is in storage form, b float32 or None."""
    y = x @ widen(W, dtype).T
    if b is not None:
        y = y + np.asarray(b, np.float64)
    return y


def layer_norm(z: np.ndarray, g, b, eps: float = LN_EPS) -> np.ndarray:
    """Per row: (z - mean) / sqrt(var + eps) * g + b, biased variance."""
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    return (z - mu) / np.sqrt(var + eps) * np.asarray(g, np.float64) + np.asarray(b, np.float64)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, heads: int = HEADS) -> np.ndarray:
    """Multi-head softmax(q k^T / sqrt(dh)) v over all rows given (one sequence's image tokens)."""
    n, c = q.shape
    dh = c // heads
    out = np.empty_like(q)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(dh)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        out[:, sl] = (p @ v[:, sl]) / p.sum(axis=1, keepdims=True)
    return out


def vit_block(z: np.ndarray, span_off, blk: Dict[str, np.ndarray], dtype: str, rnd: bool) -> np.ndarray:
    """One pre-norm transformer block over the rows z [M, 512]; rows span_off[b]..span_off[b+1] mix."""
    y = _stored(layer_norm(z, blk["ln1_g"], blk["ln1_b"]), dtype, rnd)
    qkv = _stored(linear(y, blk["Wqkv"], blk["bqkv"], dtype), dtype, rnd)
    a = np.empty_like(z)
    for b in range(len(span_off) - 1):
        r0, r1 = int(span_off[b]), int(span_off[b + 1])
        if r1 > r0:
            a[r0:r1] = attention(qkv[r0:r1, :WIDTH], qkv[r0:r1, WIDTH:2 * WIDTH], qkv[r0:r1, 2 * WIDTH:])
    a = _stored(a, dtype, rnd)
    z = _stored(z + linear(a, blk["Wo"], blk["bo"], dtype), dtype, rnd)
    y = _stored(layer_norm(z, blk["ln2_g"], blk["ln2_b"]), dtype, rnd)
    hdn = _stored(gelu(linear(y, blk["Wfc1"], blk["bfc1"], dtype)), dtype, rnd)
    return _stored(z + linear(hdn, blk["Wfc2"], blk["bfc2"], dtype), dtype, rnd)


def predict(x, span_off: Optional[np.ndarray], P: Dict, dtype: str, round_intermediates: bool = True) -> np.ndarray:
    """Logits D [M, 2] (float32) of the rows x [M, d] (storage form).

    P["blocks"] is the list of transformer blocks (two for the image predictor, empty for the output-text
    predictor).  span_off [B+1] cuts the rows into the image-token spans that attend to one another; it is
    ignored (may be None) when there are no blocks.
    """
    rnd = round_intermediates
    z = _stored(linear(widen(x, dtype), P["W_in"], P["b_in"], dtype), dtype, rnd)
    for blk in P["blocks"]:
        z = vit_block(z, span_off, blk, dtype, rnd)
    h1 = _stored(gelu(linear(z, P["W_h1"], P["b_h1"], dtype)), dtype, rnd)
    h2 = _stored(gelu(linear(h1, P["W_h2"], P["b_h2"], dtype)), dtype, rnd)
    return linear(h2, P["W_h3"], P["b_h3"], dtype).astype(np.float32)


def predict_flops(M: int, d: int, span_lens, n_blocks: int) -> float:
    """Multiply-add flops (2 per MAC) of predict(): linear layers plus the two attention products."""
    lin = 2.0 * M * (d * WIDTH + WIDTH * 256 + 256 * 128 + 128 * 2)
    per_block = 2.0 * M * (3 * WIDTH * WIDTH + WIDTH * WIDTH + 2 * WIDTH * MLP_WIDTH)
    att = sum(4.0 * n * n * WIDTH for n in span_lens)
    return lin + n_blocks * (per_block + att)
