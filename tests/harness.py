"""Shared plumbing of the GPU parity tests: moves the seeded inputs to the device and drives the
library through its Python binding.  No arithmetic of the method happens here."""
from __future__ import annotations

import math

import numpy as np
import torch

import paper_2412_00876_amd as P
from synth import workloads as W

DEV = "cuda:0"


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> stored numpy form (uint16 bit patterns for bfloat16)."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def as_f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class GpuPath:
    """One workload resident on the GPU, with its cache and workspaces."""

    def __init__(self, w: W.Workload, pre=None, pred=None, extra_tokens=0, n_pages=None, bt=None):
        self.w = w
        self.code = P.BF16 if w.dtype == "bf16" else P.F32
        td = tdtype(w.dtype)
        i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(DEV)
        self.seq_off, self.vis_start, self.vis_len = i32(w.seq_off), i32(w.vis_start), i32(w.vis_len)
        if bt is None:
            bt, n_pages = W.block_table(w, extra_tokens=extra_tokens)
        self.bt_np = bt
        self.pages = torch.zeros((n_pages, 2, w.H, 16, w.Dh), dtype=td, device=DEV)
        self.cache_len = torch.zeros(w.B, dtype=torch.int32, device=DEV)
        self.cache = P.KVCache(self.pages, i32(bt), self.cache_len)
        self.err = torch.zeros(1, dtype=torch.int32, device=DEV)
        self.pre = {k: to_dev(v, w.dtype) for k, v in pre.items()} if pre else None
        self.pred = None
        if pred:
            self.pred = {"W1": to_dev(pred["W1"], w.dtype), "W2": to_dev(pred["W2"], w.dtype),
                         "b1": to_dev(pred["b1"], "f32"), "b2": to_dev(pred["b2"], "f32")}
        # one zero-filled workspace per entry point (their counters must start at zero and stay private)
        z = lambda n: torch.zeros(n, dtype=torch.uint8, device=DEV)
        self.ws_select = z(P.dllava_select_compact_workspace(w.B, w.sumN))
        self.ws_decode = z(P.dllava_decode_workspace(w.B, w.H, w.Dh, self.cache.max_pages_per_seq))
        self.ws_score = z(P.dllava_score_workspace(max(w.sumN, w.B, 1), w.d, w.dh, self.code))
        self.ws_score_small = z(P.dllava_score_workspace(64, w.d, w.dh, self.code))
        self.scale = 1.0 / math.sqrt(w.Dh)

    # -- steps ------------------------------------------------------------------------------
    def score_vision(self) -> torch.Tensor:
        w = self.w
        M = int(sum(w.n_vis))
        logits = torch.full((M, 2), float("nan"), dtype=torch.float32, device=DEV)
        p = self.pred
        P.dllava_score(self.pre["hidden"], w.d, M, w.B, self.seq_off, self.vis_start, self.vis_len, w.d, w.dh,
                       p["W1"], p["b1"], p["W2"], p["b2"], self.code, logits, self.ws_score)
        return logits

    def score_rows(self, x: torch.Tensor) -> torch.Tensor:
        w = self.w
        M = x.shape[0]
        logits = torch.full((M, 2), float("nan"), dtype=torch.float32, device=DEV)
        p = self.pred
        P.dllava_score(x, x.stride(0), M, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"],
                       self.code, logits, self.ws_score_small if M <= 64 else self.ws_score)
        return logits

    def select_compact(self, logits: torch.Tensor, mode=P.MODE_TOPK, ratio=None, theta=0.0,
                       with_hidden=True, with_q=True, with_kv=True):
        w = self.w
        ratio = w.keep_ratio if ratio is None else ratio
        td = tdtype(w.dtype)
        sumN = w.sumN
        out = {
            "keep_mask": torch.full((sumN,), 255, dtype=torch.uint8, device=DEV),
            "kept_idx": torch.full((sumN,), -1, dtype=torch.int32, device=DEV),
            "out_off": torch.full((w.B + 1,), -1, dtype=torch.int32, device=DEV),
            "hidden_out": torch.zeros((sumN, w.d), dtype=td, device=DEV) if with_hidden else None,
            "Q_out": torch.zeros((sumN, w.H, w.Dh), dtype=td, device=DEV) if with_q else None,
        }
        pre = self.pre
        P.dllava_select_compact(logits, w.B, self.seq_off, self.vis_start, self.vis_len, sumN, mode, ratio, theta,
                                pre["hidden"] if with_hidden else None, out["hidden_out"], w.d,
                                pre["Q"] if with_q else None, out["Q_out"],
                                pre["K"] if with_kv else None, pre["V"] if with_kv else None,
                                self.cache if (with_kv or with_q) else None,
                                out["keep_mask"], out["kept_idx"], out["out_off"], self.err, self.code, self.ws_select)
        return out

    def prefill(self, Qc: torch.Tensor, off: torch.Tensor, K=None, V=None) -> torch.Tensor:
        w = self.w
        O = torch.zeros_like(Qc)
        P.dllava_prefill_attn(Qc, K, V, self.cache if K is None else None, w.B, off, Qc.shape[0], w.H, w.Dh,
                              self.scale, O, self.code)
        return O

    def decode(self, q, k, v, logits=None, theta=0.0, keep_override=None):
        w = self.w
        o = torch.zeros_like(q)
        keep = torch.full((w.B,), 255, dtype=torch.uint8, device=DEV)
        P.dllava_decode_attn_append(q, k, v, w.B, logits, theta, keep_override, self.cache, self.scale, o, keep,
                                    self.err, self.ws_decode)
        return o, keep

    def cache_rows(self, b: int, L: int):
        """K, V rows [L,H,Dh] of sequence b read back from the pages (stored form)."""
        pg = bits(self.pages)
        K = np.empty((L, self.w.H, self.w.Dh), pg.dtype)
        V = np.empty_like(K)
        for t in range(L):
            p, s = int(self.bt_np[b, t // 16]), t % 16
            K[t], V[t] = pg[p, 0, :, s, :], pg[p, 1, :, s, :]
        return K, V
