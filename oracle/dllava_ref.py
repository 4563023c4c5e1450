"""CPU oracle for the sparsify-then-attend path of Dynamic-LLaVA.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct statement
of what the GPU library must compute, written from the paper (Sec. 3.3.2,
Eq. 5, 6, 7 and Appendix A.1, Eq. 11) with numpy in float64.  Only the tests,
the smoke check and the benchmark's ``cpu_baseline`` leg may import it; the
product path never does, and it shares no code with the HIP kernels.

Conventions
  * Stored tensors arrive either as float32 arrays ("f32") or as uint16
    bfloat16 bit patterns ("bf16"); they are widened exactly and all
    arithmetic is float64.  Logits leave ``score`` rounded to float32, and
    every keep decision is taken on those float32 logits in float32, which is
    the precision the GPU path decides in.
  * Predictor (simplified two-layer form fixed by the benchmark definition,
    standing in for the MLPs of Appendix A.4.1): D = GELU(x W1^T + b1) W2^T + b2,
    exact (erf) GELU.  Column 0 of D is "drop", column 1 is "keep" (Eq. 5:
    a token is kept when the second value exceeds the first).
  * Vision tokens: per sequence keep the k = floor(r * n_vis) tokens with the
    largest D[:, 1] (Eq. 11); ties go to the lower index; NaN ranks below
    every number; -0 == +0.  Text tokens are always kept in prefill.
  * Kept tokens stay in their original order, so causal attention over the
    compacted sequence equals masked causal attention over the full one (Eq. 7).
  * Decode (Eq. 6): the new token always takes part in its own attention;
    its K/V enter the cache only when its keep decision is 1.
  * Paged cache layout: pages[n_pages][2 (K,V)][H][page_size][Dh]; token t of
    sequence b lives in page block_table[b, t // page_size], slot t % page_size.

  * Training form (Eq. 7): the same attention on the full token set with the mask inside the softmax;
    ``masked_attn`` is that definition written out, every row (kept or not) gets an output.

  * Projection of the reduced set (Eq. 3, first line, applied to S^{P*}): Q, K, V
    of the kept rows only; queries and keys optionally rotated by the ORIGINAL
    position of each kept token (rotary embedding of the LLaMA decoder).

Parity unpinned (fixed by the benchmark definition, nothing in the paper can
confirm them): the two-layer predictor shape and its GELU variant, ranking by
the raw keep logit rather than the margin, the tie-break direction, the
threshold value and the weight initialisation; the rotary convention, its base
and the use of original positions (the paper does not mention positions).
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

TOPK = 0
THRESHOLD = 1
THRESHOLD_KEEP_LAST = 2   # Sec. 3.3.2, decoding without KV cache: the mask entry of the last output token is 1


# ----------------------------------------------------------------------------- storage

def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values -> float64, exactly."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        bits = np.asarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def narrow(a: np.ndarray, dtype: str) -> np.ndarray:
    """float64 values -> stored form: float32, or bfloat16 bit patterns rounded to nearest even."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return f
    if dtype == "bf16":
        u = np.ascontiguousarray(f).view(np.uint32)
        r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        out = (r >> np.uint32(16)).astype(np.uint16)
        nan = np.isnan(f)
        if nan.any():
            out = np.where(nan, np.uint16(0x7FC0), out)
        return out
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- Eq. 5 line 1 / Eq. 11 line 1

def gelu(a: np.ndarray) -> np.ndarray:
    return 0.5 * a * (1.0 + _erf(a / math.sqrt(2.0)))


def score(x, W1, b1, W2, b2, dtype: str) -> np.ndarray:
    """Predictor logits D [M,2] (float32) for rows x [M,d]."""
    xf = widen(x, dtype)
    a = xf @ widen(W1, dtype).T
    if b1 is not None:
        a = a + np.asarray(b1, np.float64)
    h = gelu(a)
    D = h @ widen(W2, dtype).T
    if b2 is not None:
        D = D + np.asarray(b2, np.float64)
    return D.astype(np.float32)


# ----------------------------------------------------------------------------- Eq. 11 line 2, Eq. 5 line 2

def keep_count(keep_ratio: float, n_vis: int) -> int:
    """k = floor(r^I * |S^I|), evaluated in float64."""
    return int(math.floor(float(keep_ratio) * float(n_vis)))


def select_topk(scores: np.ndarray, k: int) -> np.ndarray:
    """Indices (ascending) of the k largest float32 scores; ties -> lower index; NaN lowest."""
    s = np.asarray(scores, dtype=np.float32)
    n = s.shape[0]
    k = max(0, min(int(k), n))

    def key(i):
        v = float(s[i])
        if v != v:
            return (1, 0.0, i)
        return (0, -v, i)          # -(-0.0) == 0.0 == -(+0.0): equal keys, index decides

    order = sorted(range(n), key=key)
    return np.array(sorted(order[:k]), dtype=np.int32)


def select_threshold(logits: np.ndarray, theta: float) -> np.ndarray:
    """keep = (D[:,1] - D[:,0] > theta), strict, in float32."""
    D = np.asarray(logits, dtype=np.float32)
    margin = (D[:, 1] - D[:, 0]).astype(np.float32)
    return (margin > np.float32(theta)).astype(np.uint8)


def select(logits, seq_off, vis_start, vis_len, mode: int, keep_ratio: float, theta: float):
    """Keep decisions for a ragged batch.

    logits [sum(vis_len), 2] holds the vision rows of all sequences back to back.
    Returns keep_mask [sumN] u8, kept_idx [sum N*] i32 (sequence-relative original
    positions, ascending within a sequence) and out_off [B+1] i32.
    """
    seq_off = np.asarray(seq_off)
    B = len(seq_off) - 1
    D = np.asarray(logits, dtype=np.float32).reshape(-1, 2)
    keep_mask = np.ones(int(seq_off[-1]), dtype=np.uint8)
    kept, out_off, lo = [], [0], 0
    for b in range(B):
        n, v0 = int(vis_len[b]), int(vis_start[b])
        Db = D[lo:lo + n]
        lo += n
        if mode == TOPK:
            m = np.zeros(n, np.uint8)
            m[select_topk(Db[:, 1], keep_count(keep_ratio, n))] = 1
        elif mode == THRESHOLD:
            m = select_threshold(Db, theta)
        elif mode == THRESHOLD_KEEP_LAST:
            m = select_threshold(Db, theta)
            if n:
                m[n - 1] = 1
        else:
            raise ValueError(mode)
        base = int(seq_off[b])
        keep_mask[base + v0: base + v0 + n] = m
        idx = np.nonzero(keep_mask[base:int(seq_off[b + 1])])[0].astype(np.int32)
        kept.append(idx)
        out_off.append(out_off[-1] + len(idx))
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, np.int32)
    return keep_mask, kept_idx.astype(np.int32), np.array(out_off, dtype=np.int32)


# ----------------------------------------------------------------------------- Eq. 5 line 3 / Eq. 11 line 3

class PagedCache:
    """Caller-owned paged KV cache of one layer (stored dtype, raw bits for bf16)."""

    def __init__(self, n_pages, block_table, H, Dh, dtype, page_size=16):
        self.dtype = dtype
        self.page_size = page_size
        self.H, self.Dh = H, Dh
        self.block_table = np.asarray(block_table, dtype=np.int32)
        st = np.float32 if dtype == "f32" else np.uint16
        self.pages = np.zeros((n_pages, 2, H, page_size, Dh), dtype=st)
        self.cache_len = np.zeros(self.block_table.shape[0], dtype=np.int32)

    @property
    def capacity(self) -> int:
        return self.block_table.shape[1] * self.page_size

    def put(self, b, t, k_row, v_row):
        pg = int(self.block_table[b, t // self.page_size])
        sl = t % self.page_size
        self.pages[pg, 0, :, sl, :] = k_row
        self.pages[pg, 1, :, sl, :] = v_row

    def rows(self, b, L=None):
        """K, V of sequence b as [L,H,Dh] stored-dtype arrays."""
        L = int(self.cache_len[b]) if L is None else L
        K = np.empty((L, self.H, self.Dh), self.pages.dtype)
        V = np.empty_like(K)
        for t in range(L):
            pg = int(self.block_table[b, t // self.page_size])
            sl = t % self.page_size
            K[t] = self.pages[pg, 0, :, sl, :]
            V[t] = self.pages[pg, 1, :, sl, :]
        return K, V


def compact(kept_idx, out_off, seq_off, hidden=None, Q=None, K=None, V=None, cache: Optional[PagedCache] = None):
    """Gather kept rows, order preserved.  Returns (hidden*, Q*) and fills the cache."""
    B = len(out_off) - 1
    src = np.concatenate([int(seq_off[b]) + kept_idx[out_off[b]:out_off[b + 1]] for b in range(B)]) \
        if B else np.zeros(0, np.int64)
    h_out = None if hidden is None else np.ascontiguousarray(hidden[src])
    q_out = None if Q is None else np.ascontiguousarray(Q[src])
    if cache is not None:
        for b in range(B):
            n = int(out_off[b + 1] - out_off[b])
            if n > cache.capacity:
                raise ValueError("cache capacity exceeded")
            for t in range(n):
                r = src[out_off[b] + t]
                cache.put(b, t, K[r], V[r])
            cache.cache_len[b] = n
    return h_out, q_out


# ----------------------------------------------------------------------------- Eq. 1 over the reduced set

def _softmax_av(s: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(s) @ v for one query: s [L], v [L,Dh] (float64)."""
    p = np.exp(s - s.max())
    return (p @ v) / p.sum()


def prefill_attn(Q, K, V, off, scale: float, dtype: str) -> np.ndarray:
    """Causal scaled-dot-product attention per sequence and head over compacted rows.

    Q,K,V [sum N*,H,Dh] stored dtype; returns O [sum N*,H,Dh] float64.
    """
    Qf, Kf, Vf = widen(Q, dtype), widen(K, dtype), widen(V, dtype)
    O = np.zeros_like(Qf)
    for b in range(len(off) - 1):
        r0, r1 = int(off[b]), int(off[b + 1])
        for h in range(Qf.shape[1]):
            q, k, v = Qf[r0:r1, h], Kf[r0:r1, h], Vf[r0:r1, h]
            S = (q @ k.T) * scale
            for i in range(r1 - r0):
                O[r0 + i, h] = _softmax_av(S[i, : i + 1], v[: i + 1])
    return O


# ----------------------------------------------------------------------------- Eq. 6

def masked_attn(Q, K, V, off, keep, scale: float, dtype: str) -> np.ndarray:
    """Attention of the end-to-end sparsification training (Sec. 3.3.3, Eq. 7) on the FULL token set.

    Per sequence and head, with X = scale * Q K^T: weights exp(X_ij) G_ij / sum_k exp(X_ik) G_ik, where
    G_ij = keep[j] for j < i, G_ii = 1 (the diagonal is set to one), and G_ij = 0 for j > i (the decoder's causal
    order).  Every row gets an output, also the rows whose own mask entry is 0.  Returns O [rows, H, Dh] float64.
    """
    Qf, Kf, Vf = widen(Q, dtype), widen(K, dtype), widen(V, dtype)
    keep = np.asarray(keep).astype(bool)
    O = np.zeros(Qf.shape, dtype=np.float64)
    for b in range(len(off) - 1):
        r0, r1 = int(off[b]), int(off[b + 1])
        n = r1 - r0
        if n == 0:
            continue
        G = np.tril(np.broadcast_to(keep[r0:r1][None, :], (n, n)) | np.eye(n, dtype=bool))
        for h in range(Qf.shape[1]):
            x = (Qf[r0:r1, h] @ Kf[r0:r1, h].T) * scale
            x = np.where(G, x, -np.inf)
            e = np.exp(x - x.max(axis=1, keepdims=True)) * G
            O[r0:r1, h] = (e @ Vf[r0:r1, h]) / e.sum(axis=1, keepdims=True)
    return O


def masked_attn_rows(Q, K, V, off, keep, scale: float, dtype: str, rows) -> np.ndarray:
    """Rows `rows` (global row numbers) of masked_attn, one by one, for sequences too long for the dense form."""
    off = np.asarray(off)
    keep = np.asarray(keep).astype(bool)
    out = np.zeros((len(rows),) + tuple(np.shape(Q)[1:]), dtype=np.float64)
    for n_out, i in enumerate(rows):
        b = int(np.searchsorted(off, i, side="right") - 1)
        r0 = int(off[b])
        q = widen(Q[i], dtype)
        Kf, Vf = widen(K[r0:i + 1], dtype), widen(V[r0:i + 1], dtype)
        g = keep[r0:i + 1].copy()
        g[-1] = True                                   # diag(G) = 1
        for h in range(q.shape[0]):
            x = (Kf[:, h] @ q[h]) * scale
            e = np.exp(x - x[g].max()) * g
            out[n_out, h] = (e @ Vf[:, h]) / e.sum()
    return out


def decode_keep(logits, theta, keep_override=None) -> np.ndarray:
    if keep_override is not None:
        return (np.asarray(keep_override) != 0).astype(np.uint8)
    return select_threshold(logits, theta)


def decode_attn_append(q, k_new, v_new, keep, cache: PagedCache, scale: float,
                       only: Optional[Sequence[Tuple[int, int]]] = None):
    """One decode step for a batch.

    q,k_new,v_new [B,H,Dh] stored dtype; keep [B] u8.  Attention runs over the
    cached rows followed by the new token; afterwards the new K/V are appended
    where keep is 1 (skipped, and flagged, if the sequence is at capacity).
    Returns (o [B,H,Dh] float64, err [B] u8).  ``only`` restricts the attention
    outputs to the listed (b,h) pairs (the rest stay zero); appends always happen.
    """
    dt = cache.dtype
    B, H, Dh = q.shape
    qf, kf, vf = widen(q, dt), widen(k_new, dt), widen(v_new, dt)
    o = np.zeros((B, H, Dh), np.float64)
    err = np.zeros(B, np.uint8)
    pairs = only if only is not None else [(b, h) for b in range(B) for h in range(H)]
    by_b = {}
    for b, h in pairs:
        by_b.setdefault(b, []).append(h)
    for b, hs in by_b.items():
        Kc, Vc = cache.rows(b)
        Kc, Vc = widen(Kc, dt), widen(Vc, dt)
        for h in hs:
            k = np.concatenate([Kc[:, h], kf[b, h][None]], axis=0)
            v = np.concatenate([Vc[:, h], vf[b, h][None]], axis=0)
            o[b, h] = _softmax_av((k @ qf[b, h]) * scale, v)
    for b in range(B):
        if keep[b]:
            L = int(cache.cache_len[b])
            if L >= cache.capacity:
                err[b] = 1
                continue
            cache.put(b, L, k_new[b], v_new[b])
            cache.cache_len[b] = L + 1
    return o, err


# ----------------------------------------------------------------------------- Sec. 3.3.2 / Eq. 12: decoding without KV cache

def decode_nocache_step(Qp, Kp, Vp, p_off, Qo, Ko, Vo, o_off, logits_ot, theta: float, scale: float, dtype: str):
    """One decoding step WITHOUT KV cache for a batch.

    Sequence b consists of its reduced prompt S^{P*}(b) (rows p_off[b]:p_off[b+1] of Qp/Kp/Vp) followed by ALL its
    output text tokens so far (rows o_off[b]:o_off[b+1] of Qo/Ko/Vo, logits_ot [sum n_ot, 2] their predictor
    logits).  The output tokens are masked by the threshold rule with the last one kept regardless (it generates
    the next token), the kept rows are compacted in order, and causal attention (Eq. 1) runs over S^{P*} u S^{OT*}.
    Returns (O [sum kept rows, H, Dh], out_off [B+1], keep_mask over the concatenated sequences).
    """
    B = len(p_off) - 1
    n_p = [int(p_off[b + 1] - p_off[b]) for b in range(B)]
    n_o = [int(o_off[b + 1] - o_off[b]) for b in range(B)]
    cat = lambda P_, O_: np.concatenate([np.concatenate([P_[p_off[b]:p_off[b + 1]], O_[o_off[b]:o_off[b + 1]]])
                                         for b in range(B)]) if B else P_[:0]
    Q, K, V = cat(Qp, Qo), cat(Kp, Ko), cat(Vp, Vo)
    seq_off = np.concatenate([[0], np.cumsum([n_p[b] + n_o[b] for b in range(B)])]).astype(np.int64)
    mask, idx, off = select(logits_ot, seq_off, n_p, n_o, THRESHOLD_KEEP_LAST, 0.0, theta)
    src = np.concatenate([seq_off[b] + idx[off[b]:off[b + 1]] for b in range(B)]) if B else np.zeros(0, np.int64)
    O = prefill_attn(Q[src], K[src], V[src], off, scale, dtype)
    return O, off, mask


# ----------------------------------------------------------------------------- Eq. 3 line 1 over the reduced set

def rope_rotate(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary position embedding of x [n,H,Dh] at integer positions pos [n] (float64).

    The decoder the paper sparsifies is LLaMA-style; its attention rotates queries and keys by position before the
    dot product (RoFormer; the pairing used by LLaMA: feature i goes with feature i + Dh/2, angle
    pos * base^(-2i/Dh)).  The paper never mentions positions (parity unpinned: the convention and the use of the
    ORIGINAL positions of the kept tokens are this library's reading).
    """
    n, H, Dh = x.shape
    half = Dh // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / Dh)[None, :]      # [n, half]
    c, s_ = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s_, hi * c + lo * s_], axis=-1)


def qkv_project(x, off, pos, Wq, Wk, Wv, H: int, Dh: int, dtype: str, rope_base: Optional[float] = None,
                cache: Optional[PagedCache] = None):
    """Q, K, V = W^Q S, W^K S, W^V S (Eq. 3, first line) for the rows of the REDUCED set only.

    x [rows,d] are the compacted hidden states S^{P*} (Eq. 5 line 3) in stored form, off [B+1] their sequence
    offsets, pos [rows] the original sequence-relative position of every kept row (kept_idx of `select`).
    W* are [H*Dh, d] stored.  Queries and keys are rotated (rope_rotate) when rope_base is given.
    Returns float64 Q, K, V [rows,H,Dh]; when a cache is given, K and V are rounded to its stored form and
    written at positions 0..n_b-1 of every sequence, and cache_len[b] = n_b.
    """
    xs = widen(x, dtype)
    rows = xs.shape[0]
    out = []
    for W in (Wq, Wk, Wv):
        out.append((xs @ widen(W, dtype).T).reshape(rows, H, Dh))
    Q, K, V = out
    if rope_base is not None:
        Q = rope_rotate(Q, pos, rope_base)
        K = rope_rotate(K, pos, rope_base)
    if cache is not None:
        Ks, Vs = narrow(K, dtype), narrow(V, dtype)
        B = len(off) - 1
        for b in range(B):
            n = int(off[b + 1] - off[b])
            if n > cache.capacity:
                raise ValueError("cache capacity exceeded")
            for t in range(n):
                cache.put(b, t, Ks[off[b] + t], Vs[off[b] + t])
            cache.cache_len[b] = n
    return Q, K, V


# ----------------------------------------------------------------------------- Appendix A.4.2, Eq. 13

def prefill_flops_eq13(n_tokens: int, C: int, batch: int = 1) -> float:
    """Per-layer prefill FLOPs of the image tokens: 32 B N C^2 + 4 B N^2 C."""
    return 32.0 * batch * n_tokens * C * C + 4.0 * batch * n_tokens * n_tokens * C


def model_prefill_tflops(n_full: int, n_kept: int, C: int, layers: int, sparsify_after: int) -> float:
    """Image-token prefill TFLOPs when layers 1..sparsify_after see n_full tokens and the rest n_kept."""
    f = sparsify_after * prefill_flops_eq13(n_full, C) + (layers - sparsify_after) * prefill_flops_eq13(n_kept, C)
    return f / 1e12
