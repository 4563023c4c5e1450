"""Seeded synthetic workloads with the shapes of LLaVA-1.5 sparsified inference.

The shapes stand in for the paper's evaluation workloads (576 image tokens per
picture, tens to hundreds of prompt tokens, hundreds to thousands of generated
tokens, batch 1 to 32).  No dataset item is reproduced: every tensor is drawn
from the counter-based streams in ``synth.rng``.

Floating tensors are returned in the workload's storage type: ``float32``
arrays for "f32", ``uint16`` bit patterns (bfloat16, round-to-nearest-even of
the float32 draw) for "bf16".  Both the CPU oracle and the GPU path are fed
these same bytes.  Nothing here computes any part of the sparsification method;
the optional Q/K/V projection is the decoder layer's own linear map, which lies
outside the method's hot path and only shapes the inputs.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Sequence

import numpy as np

from . import rng

PAGE_SIZE = 16


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def stored_to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    """Widen stored values back to float32 (exact)."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32)
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    d: int                     # hidden size
    H: int                     # attention heads
    Dh: int                    # head dim
    dh: int                    # predictor hidden width (d/4)
    n_sys: Sequence[int]       # per sequence
    n_vis: Sequence[int]
    n_prompt: Sequence[int]
    keep_ratio: float          # r^I, vision keep ratio
    T: int                     # decode steps
    theta: float = 0.0         # text keep threshold on the logit margin
    project_qkv: bool = False  # Q/K/V = hidden @ W^T (else drawn directly)
    seed: int = 0x0D11A5A0
    page_size: int = PAGE_SIZE

    @property
    def B(self) -> int:
        return len(self.n_vis)

    @property
    def seq_len(self) -> List[int]:
        return [a + b + c for a, b, c in zip(self.n_sys, self.n_vis, self.n_prompt)]

    @property
    def seq_off(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_len)]).astype(np.int32)

    @property
    def vis_start(self) -> np.ndarray:
        return np.asarray(self.n_sys, dtype=np.int32)

    @property
    def vis_len(self) -> np.ndarray:
        return np.asarray(self.n_vis, dtype=np.int32)

    @property
    def k_keep(self) -> List[int]:
        return [int(math.floor(float(self.keep_ratio) * float(n))) for n in self.n_vis]

    @property
    def kept_len(self) -> List[int]:
        return [a + k + c for a, k, c in zip(self.n_sys, self.k_keep, self.n_prompt)]

    @property
    def sumN(self) -> int:
        return int(sum(self.seq_len))

    def max_pages_per_seq(self, extra_tokens: int = 0) -> int:
        cap = max(self.kept_len) + self.T + extra_tokens
        return (cap + self.page_size - 1) // self.page_size


def _rep(v, B):
    return [int(v)] * B if np.isscalar(v) else [int(x) for x in v]


def make(name, dtype, d, H, Dh, B, n_sys, n_vis, n_prompt, keep_ratio, T, **kw) -> Workload:
    return Workload(name=name, dtype=dtype, d=d, H=H, Dh=Dh, dh=d // 4,
                    n_sys=_rep(n_sys, B), n_vis=_rep(n_vis, B), n_prompt=_rep(n_prompt, B),
                    keep_ratio=keep_ratio, T=T, **kw)


def config(i: int) -> Workload:
    """The five benchmark configurations, by index 0..4 (C1..C5)."""
    s = 0x0D11A5A0 + i
    if i == 0:   # tiny fp32 layer
        return make("C1-tiny-f32", "f32", 512, 8, 64, 1, 16, 64, 16, 0.25, 8, project_qkv=True, seed=s)
    if i == 1:   # LLaVA-1.5-7B shaped single layer, batch 1
        return make("C2-7B-b1", "bf16", 4096, 32, 128, 1, 35, 576, 64, 0.2, 256, project_qkv=True, seed=s)
    if i == 2:   # 7B decode-heavy: the C2 prompt shape, batch 16, 1024 generated tokens
        return make("C3-7B-decode-b16", "bf16", 4096, 32, 128, 16, 35, 576, 64, 0.2, 1024, seed=s)
    if i == 3:   # 13B shaped, batch 32
        return make("C4-13B-b32", "bf16", 5120, 40, 128, 32, 0, 576, 128, 0.2, 512, seed=s)
    if i == 4:   # high-resolution, 5 tiles of 576 vision tokens, batch 8
        return make("C5-anyres-b8", "bf16", 4096, 32, 128, 8, 0, 2880, 128, 0.2, 2048, seed=s)
    raise IndexError(i)


# --------------------------------------------------------------------------- tensors

def _xavier(seed, name, fan_out, fan_in):
    a = math.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(seed, name, (fan_out, fan_in), -a, a).astype(np.float32)


def _normal_big(seed, name, shape, threads=8):
    """rng.normal, with the leading axis cut into slabs drawn by a thread pool.

    Slab j of a tensor uses the sub-stream "<name>#j", so the values depend on
    the slab size (fixed below) but not on the number of threads.
    """
    n = int(np.prod(shape))
    if n <= (1 << 22):
        return rng.normal(seed, name, shape)
    lead = shape[0]
    per = max(1, (1 << 22) // max(1, n // lead))
    jobs = [(j, r0, min(lead, r0 + per)) for j, r0 in enumerate(range(0, lead, per))]
    out = np.empty(shape, dtype=np.float32)

    def run(job):
        j, r0, r1 = job
        out[r0:r1] = rng.normal(seed, f"{name}#{j}", (r1 - r0,) + tuple(shape[1:]))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(run, jobs))
    return out


def predictor(w: Workload, random_bias: bool = False) -> Dict[str, np.ndarray]:
    """Two-layer predictor d -> d/4 -> 2, Xavier-uniform weights; W in storage dtype, biases float32."""
    W1 = _xavier(w.seed, "pred.W1", w.dh, w.d)
    W2 = _xavier(w.seed, "pred.W2", 2, w.dh)
    if random_bias:
        b1 = rng.uniform(w.seed, "pred.b1", (w.dh,), -0.5, 0.5).astype(np.float32)
        b2 = rng.uniform(w.seed, "pred.b2", (2,), -0.5, 0.5).astype(np.float32)
    else:
        b1 = np.zeros(w.dh, np.float32)
        b2 = np.zeros(2, np.float32)
    return {"W1": store(W1, w.dtype), "b1": b1, "W2": store(W2, w.dtype), "b2": b2}


def paper_predictor(w: Workload, n_blocks: int, name: str = "ppred") -> Dict:
    """Weights of a predictor in the appendix's form (Appendix A.4.1): d -> 512, n_blocks transformer blocks
    (width 512, MLP 2048), head 512 -> 256 -> 128 -> 2.  Xavier-uniform matrices in storage dtype; float32
    biases in [-0.1, 0.1], LayerNorm scales in [0.9, 1.1] and shifts in [-0.1, 0.1] (all seeded)."""
    def mat(tag, fo, fi):
        return store(_xavier(w.seed, f"{name}.{tag}", fo, fi), w.dtype)

    def vec(tag, n, lo=-0.1, hi=0.1):
        return rng.uniform(w.seed, f"{name}.{tag}", (n,), lo, hi).astype(np.float32)

    P = {"W_in": mat("W_in", 512, w.d), "b_in": vec("b_in", 512), "blocks": []}
    for i in range(n_blocks):
        t = f"blk{i}."
        P["blocks"].append({
            "ln1_g": vec(t + "ln1_g", 512, 0.9, 1.1), "ln1_b": vec(t + "ln1_b", 512),
            "Wqkv": mat(t + "Wqkv", 1536, 512), "bqkv": vec(t + "bqkv", 1536),
            "Wo": mat(t + "Wo", 512, 512), "bo": vec(t + "bo", 512),
            "ln2_g": vec(t + "ln2_g", 512, 0.9, 1.1), "ln2_b": vec(t + "ln2_b", 512),
            "Wfc1": mat(t + "Wfc1", 2048, 512), "bfc1": vec(t + "bfc1", 2048),
            "Wfc2": mat(t + "Wfc2", 512, 2048), "bfc2": vec(t + "bfc2", 512),
        })
    P["W_h1"], P["b_h1"] = mat("W_h1", 256, 512), vec("b_h1", 256)
    P["W_h2"], P["b_h2"] = mat("W_h2", 128, 256), vec("b_h2", 128)
    P["W_h3"], P["b_h3"] = mat("W_h3", 2, 128), vec("b_h3", 2)
    return P


def decoder_layers(w: Workload, n_layers: int, d_ff: int, name: str = "dec") -> list:
    """Weights of n_layers LLaMA-style decoder layers (no biases): Xavier-uniform projections in storage dtype,
    RMSNorm scales in [0.8, 1.2] float32.  Keys: Wq, Wk, Wv [H*Dh, d], Wo [d, H*Dh], Wg, Wu [d_ff, d], Wd [d, d_ff], g1, g2 [d]."""
    out = []
    hd = w.H * w.Dh
    for i in range(n_layers):
        t = f"{name}.{i}."
        mat = lambda tag, fo, fi: store(_xavier(w.seed, t + tag, fo, fi), w.dtype)
        out.append({"Wq": mat("Wq", hd, w.d), "Wk": mat("Wk", hd, w.d), "Wv": mat("Wv", hd, w.d), "Wo": mat("Wo", w.d, hd),
                    "Wg": mat("Wg", d_ff, w.d), "Wu": mat("Wu", d_ff, w.d), "Wd": mat("Wd", w.d, d_ff),
                    "g1": rng.uniform(w.seed, t + "g1", (w.d,), 0.8, 1.2).astype(np.float32),
                    "g2": rng.uniform(w.seed, t + "g2", (w.d,), 0.8, 1.2).astype(np.float32)})
    return out


def _hidden(w: Workload, name: str, rows: int, unit_scale: bool) -> np.ndarray:
    g = _normal_big(w.seed, name, (rows, w.d))
    if not unit_scale:
        s = rng.uniform(w.seed, name + ".scale", (rows, 1), 0.5, 2.0).astype(np.float32)
        g *= s
    return g


def _qkv_from(w: Workload, x_stored_f32: np.ndarray):
    out = {}
    for nm in ("q", "k", "v"):
        W = _xavier(w.seed, f"attn.W{nm}", w.H * w.Dh, w.d)
        W = stored_to_f32(store(W, w.dtype), w.dtype)
        out[nm] = (x_stored_f32 @ W.T).reshape(-1, w.H, w.Dh)
    return out


def attn_weights(w: Workload) -> Dict[str, np.ndarray]:
    """Stored Xavier-uniform projection weights Wq, Wk, Wv [H*Dh, d] (the ones prefill_inputs / decode_inputs
    use when the workload projects Q/K/V from the hidden states)."""
    return {nm: store(_xavier(w.seed, f"attn.W{nm}", w.H * w.Dh, w.d), w.dtype) for nm in ("q", "k", "v")}


def prefill_inputs(w: Workload) -> Dict[str, np.ndarray]:
    """hidden [sumN,d]; Q,K,V [sumN,H,Dh] for every prompt token (before sparsification)."""
    rows = w.sumN
    unit = w.dtype == "f32"
    h = store(_hidden(w, "prefill.hidden", rows, unit), w.dtype)
    if w.project_qkv:
        qkv = _qkv_from(w, stored_to_f32(h, w.dtype))
    else:
        qkv = {nm: _normal_big(w.seed, f"prefill.{nm}", (rows, w.H, w.Dh)) for nm in ("q", "k", "v")}
    return {"hidden": h, "Q": store(qkv["q"], w.dtype), "K": store(qkv["k"], w.dtype),
            "V": store(qkv["v"], w.dtype)}


def decode_inputs(w: Workload, T: int | None = None) -> Dict[str, np.ndarray]:
    """Teacher-forced decode tokens: x [T,B,d]; q,k,v [T,B,H,Dh]."""
    T = w.T if T is None else T
    unit = w.dtype == "f32"
    x = store(_hidden(w, "decode.hidden", T * w.B, unit), w.dtype)
    if w.project_qkv:
        qkv = _qkv_from(w, stored_to_f32(x, w.dtype))
    else:
        qkv = {nm: _normal_big(w.seed, f"decode.{nm}", (T * w.B, w.H, w.Dh)) for nm in ("q", "k", "v")}
    sh = (T, w.B, w.H, w.Dh)
    return {"x": x.reshape(T, w.B, w.d), "q": store(qkv["q"], w.dtype).reshape(sh),
            "k": store(qkv["k"], w.dtype).reshape(sh), "v": store(qkv["v"], w.dtype).reshape(sh)}


def block_table(w: Workload, extra_tokens: int = 0, spare_pages: int = 0):
    """Seeded random page assignment: (block_table [B,max_pages] int32, n_pages)."""
    mp = w.max_pages_per_seq(extra_tokens)
    n_pages = w.B * mp + spare_pages
    perm = rng.permutation(w.seed, "cache.block_table", n_pages)
    return perm[: w.B * mp].reshape(w.B, mp).astype(np.int32).copy(), n_pages


def keep_pattern(w: Workload, T: int, p: float = 0.5) -> np.ndarray:
    """Seeded Bernoulli(p) keep flags [T,B] (a static random drop pattern)."""
    return rng.bernoulli(w.seed, "decode.keep_pattern", (T, w.B), p)
