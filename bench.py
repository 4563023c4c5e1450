#!/usr/bin/env python3
"""Benchmark of the sparsify-then-attend hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch:
  score vision tokens -> top-k select + compact (hidden, Q, K/V into the paged cache)
  -> causal prefill attention over the reduced set
  -> T decode steps, each: score the new tokens -> decode attention + conditional append.
The metric is generated tokens per second of that whole step (B*T tokens per step), with all
inputs resident in HBM before the timed region.  The step is recorded once into a HIP graph
(the library never synchronises with the host, cache lengths live on the device) and replayed;
`--no-graph` times the same calls issued eagerly from Python instead.

Prints ONE JSON line: metric / value / unit, the roofline object of the decode launch (algorithmic bytes per launch over
its measured duration, against the HBM peak), cpu_baseline (the oracle timed on the host on a bounded sample, per stage,
on one thread and on all cores), per-stage figures under "stages", and -- in the default run -- the same step and its
stages on the 13B (c4) and high-resolution (c5) workloads, where the matrix-core and compaction stages have their
largest shapes, and on the batch-1 prompt (batch_1).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
# HBM bytes moved per algorithmic byte by the decode kernel, from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE, each
# scaled by its reading for a 256 MiB copy): profiles/decode_attn_c3_hbm_counters.txt
DECODE_TRAFFIC_PER_ALGORITHMIC_BYTE = 1.027
# the same for the one-launch step (K+V, W1 and the hidden rows): profiles/decode_step_hbm_counters.txt
STEP_TRAFFIC_PER_ALGORITHMIC_BYTE = 1.034


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--decode-steps", type=int, default=None, help="override T (for quick runs)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--two-launch-decode", action="store_true",
                    help="decode with dllava_score + dllava_decode_attn_append (two dependent launches per step) "
                         "instead of dllava_decode_step (one launch, append deferred by one step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack", action="store_true",
                    help="also time a prefill and decode steps through 8 whole decoder layers (norms, projections, "
                         "feed-forward; 3.2 GB of random weights): outside the sparsify-then-attend path, off by default")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the stages outside the timed step (appendix-form predictors, Eq. 7 attention, decoding "
                         "without KV cache, the two-launch decode form)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="headline workload only: no c4 / c5 / batch_1 objects")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="budget of EACH of the two oracle timings (one thread, all cores)")
    ap.add_argument("--pmc-probe", type=int, default=0, metavar="L",
                    help="counter probe for rocprofv3 --pmc: one 256 MiB device copy (calibration), the prefill kernels, "
                         "3 decode launches at cache length L with appends disabled, one dispatch of each few-rows "
                         "layer of a decode step; prints the algorithmic bytes and exits")
    return ap.parse_args()


def to_dev(a: np.ndarray, dtype: str):
    """Stored numpy form (uint16 bit patterns for bfloat16) -> device tensor; plumbing only."""
    import torch
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


class Path:
    """The whole hot path for one workload, resident on the GPU."""

    def __init__(self, w, torch, P, W):
        self.to_dev = to_dev
        self.w, self.torch, self.P = w, torch, P
        dev = "cuda:0"
        self.code = P.BF16 if w.dtype == "bf16" else P.F32
        td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        t0 = time.time()
        pre = W.prefill_inputs(w)
        dec = W.decode_inputs(w)
        pred = W.predictor(w)
        self.gen_seconds = time.time() - t0
        self.host = {"pre": pre, "dec": dec, "pred": pred}
        i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(dev)
        self.seq_off, self.vis_start, self.vis_len = i32(w.seq_off), i32(w.vis_start), i32(w.vis_len)
        self.pre = {k: to_dev(v, w.dtype) for k, v in pre.items()}
        self.dec = {k: to_dev(v, w.dtype) for k, v in dec.items()}
        self.pred = {"W1": to_dev(pred["W1"], w.dtype), "W2": to_dev(pred["W2"], w.dtype),
                     "b1": to_dev(pred["b1"], "f32"), "b2": to_dev(pred["b2"], "f32")}
        bt, n_pages = W.block_table(w)
        self.bt_np = bt
        self.pages = torch.zeros((n_pages, 2, w.H, 16, w.Dh), dtype=td, device=dev)
        self.cache_len = torch.zeros(w.B, dtype=torch.int32, device=dev)
        self.cache = P.KVCache(self.pages, i32(bt), self.cache_len)
        self.err = torch.zeros(1, dtype=torch.int32, device=dev)
        sumN, T, B = w.sumN, w.T, w.B
        self.M_vis = int(sum(w.n_vis))
        self.logits_vis = torch.zeros((self.M_vis, 2), dtype=torch.float32, device=dev)
        self.keep_mask = torch.zeros(sumN, dtype=torch.uint8, device=dev)
        self.kept_idx = torch.zeros(sumN, dtype=torch.int32, device=dev)
        self.out_off = torch.zeros(B + 1, dtype=torch.int32, device=dev)
        self.rows_kept = int(sum(w.kept_len))
        self.hidden_out = torch.zeros((self.rows_kept, w.d), dtype=td, device=dev)
        self.Q_out = torch.zeros((self.rows_kept, w.H, w.Dh), dtype=td, device=dev)
        self.O = torch.zeros((self.rows_kept, w.H, w.Dh), dtype=td, device=dev)
        self.logits_dec = torch.zeros((T, B, 2), dtype=torch.float32, device=dev)
        self.o_dec = torch.zeros((T, B, w.H, w.Dh), dtype=td, device=dev)
        self.keep_dec = torch.zeros((T, B), dtype=torch.uint8, device=dev)
        z = lambda n: torch.zeros(n, dtype=torch.uint8, device=dev)
        self.attn_w = None   # projection weights of the layer: only the qkv_project stage needs them
        self.ws_score_vis = z(P.dllava_score_workspace(self.M_vis, w.d, w.dh, self.code))
        self.ws_score_dec = z(P.dllava_score_workspace(B, w.d, w.dh, self.code))
        self.ws_select = z(P.dllava_select_compact_workspace(B, sumN))
        self.ws_decode = z(P.dllava_decode_workspace(B, w.H, w.Dh, self.cache.max_pages_per_seq))
        self.ws_step = z(P.dllava_decode_step_workspace(B, w.H, w.Dh, self.cache.max_pages_per_seq, w.d, w.dh, self.code))
        self.two_launch = False
        self.scale = 1.0 / math.sqrt(w.Dh)

    def calibrate_theta(self):
        """Text keep threshold = median logit margin of this workload's decode tokens (the paper's keep
        rate r^OT = 50% is a trained property of its predictor; a random-weight predictor needs the
        threshold set to reach it).  Input preparation, outside the timed region."""
        w, p, torch = self.w, self.pred, self.torch
        x = self.dec["x"].view(-1, w.d)
        M = x.shape[0]
        ws = torch.zeros(self.P.dllava_score_workspace(M, w.d, w.dh, self.code), dtype=torch.uint8, device=x.device)
        D = torch.zeros((M, 2), dtype=torch.float32, device=x.device)
        self.P.dllava_score(x, w.d, M, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"],
                            self.code, D, ws)
        torch.cuda.synchronize()
        w.theta = float(torch.median(D[:, 1] - D[:, 0]).item())

    # ---- the stages, exactly as a caller would issue them -------------------------------------
    def score_vision(self):
        w, p = self.w, self.pred
        self.P.dllava_score(self.pre["hidden"], w.d, self.M_vis, w.B, self.seq_off, self.vis_start, self.vis_len,
                            w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], self.code, self.logits_vis,
                            self.ws_score_vis)

    def select_compact(self):
        w = self.w
        self.P.dllava_select_compact(self.logits_vis, w.B, self.seq_off, self.vis_start, self.vis_len, w.sumN,
                                     self.P.MODE_TOPK, w.keep_ratio, 0.0, self.pre["hidden"], self.hidden_out, w.d,
                                     self.pre["Q"], self.Q_out, self.pre["K"], self.pre["V"], self.cache,
                                     self.keep_mask, self.kept_idx, self.out_off, self.err, self.code, self.ws_select)

    def qkv_project(self):
        """Alternative to handing precomputed Q/K/V to select_compact: project the compacted hidden states
        (rotary rotation by original positions) straight into Q_out and the pages."""
        w = self.w
        if self.attn_w is None:
            from synth import workloads as W
            self.attn_w = {k: self.to_dev(v, w.dtype) for k, v in W.attn_weights(w).items()}
        a = self.attn_w
        self.P.dllava_qkv_project(self.hidden_out, w.d, self.rows_kept, w.d, w.B, self.out_off, self.kept_idx,
                                  a["q"], a["k"], a["v"], 10000.0, self.Q_out, self.cache, self.err, self.code)

    def prefill_attn(self):
        w = self.w
        self.P.dllava_prefill_attn(self.Q_out, None, None, self.cache, w.B, self.out_off, self.rows_kept, w.H, w.Dh,
                                   self.scale, self.O, self.code)

    def score_decode(self, t):
        w, p = self.w, self.pred
        self.P.dllava_score(self.dec["x"][t], w.d, w.B, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"],
                            p["b2"], self.code, self.logits_dec[t], self.ws_score_dec)

    def decode_attn(self, t):
        w, d = self.w, self.dec
        self.P.dllava_decode_attn_append(d["q"][t], d["k"][t], d["v"][t], w.B, self.logits_dec[t], w.theta, None,
                                         self.cache, self.scale, self.o_dec[t], self.keep_dec[t], self.err,
                                         self.ws_decode)

    def decode_step(self, t):
        """Scoring + attention of step t in one launch; the append of token t-1 happens here (deferred form)."""
        w, d, p = self.w, self.dec, self.pred
        prev = t > 0
        self.P.dllava_decode_step(d["x"][t], w.d, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"],
                                  d["q"][t], d["k"][t], d["v"][t],
                                  d["k"][t - 1] if prev else None, d["v"][t - 1] if prev else None,
                                  self.logits_dec[t - 1] if prev else None, None, w.B, w.theta, self.cache, self.scale,
                                  self.o_dec[t], self.logits_dec[t], self.keep_dec[t - 1] if prev else None, self.err,
                                  self.ws_step)

    def decode_commit(self):
        w, d, T = self.w, self.dec, self.w.T
        self.P.dllava_decode_commit(d["k"][T - 1], d["v"][T - 1], self.logits_dec[T - 1], None, w.B, w.theta, self.cache,
                                    self.keep_dec[T - 1], self.err)

    def step(self):
        self.score_vision()
        self.select_compact()
        self.prefill_attn()
        if self.two_launch:
            for t in range(self.w.T):
                self.score_decode(t)
                self.decode_attn(t)
        else:
            for t in range(self.w.T):
                self.decode_step(t)
            self.decode_commit()


class NoCacheStep:
    """One decoding step WITHOUT KV cache at the END of the generation (Sec. 3.3.2, Eq. 12): every sequence is its
    reduced prompt (kept_len rows) followed by all T output tokens; the output span is re-masked by the threshold
    rule with the last token kept, everything kept is compacted (Q, K/V into pages) and attended causally.
    Q/K/V and the output-token logits are seeded random tensors of that shape (the cost is value-independent)."""

    def __init__(self, path):
        w, P, torch = path.w, path.P, path.torch
        dev, td = "cuda:0", (torch.bfloat16 if w.dtype == "bf16" else torch.float32)
        B, T, H, Dh = w.B, w.T, w.H, w.Dh
        self.path = path
        n_p = np.asarray(w.kept_len, np.int64)
        self.seq_off_np = np.concatenate([[0], np.cumsum(n_p + T)]).astype(np.int32)
        self.sumN = int(self.seq_off_np[-1])
        i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(dev)
        self.seq_off, self.span_start, self.span_len = i32(self.seq_off_np), i32(n_p), i32([T] * B)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed + 77)
        rnd = lambda *sh: torch.randn(*sh, generator=gen, device=dev, dtype=torch.float32)
        self.Q, self.K, self.V = (rnd(self.sumN, H, Dh).to(td) for _ in range(3))
        self.logits = rnd(B * T, 2)
        mp = (int(n_p.max()) + T + 15) // 16
        self.pages = torch.zeros((B * mp, 2, H, 16, Dh), dtype=td, device=dev)
        self.cache_len = torch.zeros(B, dtype=torch.int32, device=dev)
        self.cache = P.KVCache(self.pages, i32(np.arange(B * mp).reshape(B, mp)), self.cache_len)
        self.keep_mask = torch.zeros(self.sumN, dtype=torch.uint8, device=dev)
        self.kept_idx = torch.zeros(self.sumN, dtype=torch.int32, device=dev)
        self.out_off = torch.zeros(B + 1, dtype=torch.int32, device=dev)
        self.Q_out = torch.zeros((self.sumN, H, Dh), dtype=td, device=dev)
        self.O = torch.zeros((self.sumN, H, Dh), dtype=td, device=dev)
        self.ws = torch.zeros(P.dllava_select_compact_workspace(B, self.sumN), dtype=torch.uint8, device=dev)

    def run(self):
        p, w, P = self.path, self.path.w, self.path.P
        P.dllava_select_compact(self.logits, w.B, self.seq_off, self.span_start, self.span_len, self.sumN,
                                P.MODE_THRESHOLD_KEEP_LAST, 0.0, 0.0, None, None, w.d, self.Q, self.Q_out, self.K, self.V,
                                self.cache, self.keep_mask, self.kept_idx, self.out_off, p.err, p.code, self.ws)
        P.dllava_prefill_attn(self.Q_out, None, None, self.cache, w.B, self.out_off, self.sumN, w.H, w.Dh, p.scale,
                              self.O, p.code)


class PaperPredictors:
    """The predictors in the appendix's form (Appendix A.4.1) on this workload, outside the timed step, which
    scores with the two-layer form the benchmark definition fixes: the image predictor (two transformer blocks)
    over all vision spans, and the output-text predictor over the B rows of one decode step."""

    def __init__(self, path, W):
        w, P, torch = path.w, path.P, path.torch
        dev = "cuda:0"
        self.path = path

        def desc(Pw):
            up = lambda v: path.to_dev(v, "bf16") if v.dtype == np.uint16 else torch.from_numpy(v).to(dev)
            return P.Predictor(w.d, {k: up(v) for k, v in Pw.items() if k != "blocks"},
                               [{k: up(v) for k, v in blk.items()} for blk in Pw["blocks"]])

        self.image = desc(W.paper_predictor(w, 2, "ppred.image"))
        self.text = desc(W.paper_predictor(w, 0, "ppred.text"))
        z = lambda n: torch.zeros(n, dtype=torch.uint8, device=dev)
        self.ws_image = z(P.dllava_predict_workspace(path.M_vis, w.B, 2))
        self.ws_text = z(P.dllava_predict_workspace(w.B, w.B, 0))
        self.logits_image = torch.zeros((path.M_vis, 2), dtype=torch.float32, device=dev)
        self.logits_text = torch.zeros((w.B, 2), dtype=torch.float32, device=dev)

    def run_image(self):
        p, w = self.path, self.path.w
        p.P.dllava_predict(p.pre["hidden"], w.d, p.M_vis, w.B, p.seq_off, p.vis_start, p.vis_len, self.image, p.code,
                           self.logits_image, self.ws_image)

    def run_text(self, t):
        p, w = self.path, self.path.w
        p.P.dllava_predict(p.dec["x"][t], w.d, w.B, 0, None, None, None, self.text, p.code, self.logits_text,
                           self.ws_text)

    def calibrate_theta(self):
        """Threshold of the output-text predictor = median margin over the workload's decode tokens (as for the
        two-layer predictor: the keep rate is a trained property, random weights need the threshold set)."""
        p, w, torch = self.path, self.path.w, self.path.torch
        x = p.dec["x"].view(-1, w.d)
        M = x.shape[0]
        D = torch.zeros((M, 2), dtype=torch.float32, device=x.device)
        ws = torch.zeros(p.P.dllava_predict_workspace(M, 0, 0), dtype=torch.uint8, device=x.device)
        p.P.dllava_predict(x, w.d, M, 0, None, None, None, self.text, p.code, D, ws)
        torch.cuda.synchronize()
        self.theta = float(torch.median(D[:, 1] - D[:, 0]).item())
        self.logits_steps = torch.zeros((w.T, w.B, 2), dtype=torch.float32, device=x.device)
        self.ws_attn = torch.zeros(p.P.dllava_decode_workspace(w.B, w.H, w.Dh, p.cache.max_pages_per_seq), dtype=torch.uint8,
                                   device=x.device)

    def text_step(self, t):
        p, w = self.path, self.path.w
        p.P.dllava_predict(p.dec["x"][t], w.d, w.B, 0, None, None, None, self.text, p.code, self.logits_steps[t], self.ws_text)

    def attn_step(self, t):
        """Attention + deferred append only (no scoring in the call): decisions from logits_steps[t - 1]."""
        p, w, d = self.path, self.path.w, self.path.dec
        prev = t > 0
        p.P.dllava_decode_step(None, 0, 0, 0, None, None, None, None, d["q"][t], d["k"][t], d["v"][t],
                               d["k"][t - 1] if prev else None, d["v"][t - 1] if prev else None,
                               self.logits_steps[t - 1] if prev else None, None, w.B, self.theta, p.cache, p.scale,
                               p.o_dec[t], None, None, p.err, self.ws_attn)

    def flops_image(self):
        w, M = self.path.w, self.path.M_vis
        lin = 2.0 * M * (w.d * 512 + 512 * 256 + 256 * 128 + 256) + 2 * 2.0 * M * 12 * 512 * 512
        att = 2 * sum(4.0 * n * n * 512 for n in w.n_vis)
        return lin + att


def timed_events(torch, fn, n=1):
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / n  # ms


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_pass(path, seconds, L_t):
    """One timing pass of the oracle over a bounded sample of the workload; seconds per stage, scaled to the whole step.

    Sample: the prefill stages on the first nb sequences (scaled by B / nb); the decode loop on those sequences at every
    `stride`-th step with the cache set to the EXACT length the step has in the timed run (L_t, from the GPU run's keep
    decisions; the oracle's cost depends on the lengths only), scaled by the sum of L_t over all steps."""
    from oracle import dllava_ref as R
    w, host = path.w, path.host
    pre, dec, pred = host["pre"], host["dec"], host["pred"]
    nb = min(w.B, 2)
    st = {}
    t0 = time.perf_counter()
    r1 = int(w.seq_off[nb])
    rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b]) for b in range(nb)])
    D = R.score(pre["hidden"][rows], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    t1 = time.perf_counter()
    mask, idx, off = R.select(D, w.seq_off[:nb + 1], w.vis_start[:nb], w.vis_len[:nb], R.TOPK, w.keep_ratio, 0.0)
    t2 = time.perf_counter()
    cache = R.PagedCache(path.pages.shape[0], path.bt_np[:nb], w.H, w.Dh, w.dtype)
    _, Qc = R.compact(idx, off, w.seq_off[:nb + 1], hidden=pre["hidden"][:r1], Q=pre["Q"][:r1], K=pre["K"][:r1],
                      V=pre["V"][:r1], cache=cache)
    t3 = time.perf_counter()
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(nb)])
    R.prefill_attn(Qc, pre["K"][src], pre["V"][src], off, path.scale, w.dtype)
    t4 = time.perf_counter()
    scale_pre = w.B / nb
    st["score_vision"] = (t1 - t0) * scale_pre
    st["select"] = (t2 - t1) * scale_pre
    st["compact"] = (t3 - t2) * scale_pre
    st["prefill_attn"] = (t4 - t3) * scale_pre
    # decode: the cache pages hold the prefill rows, the slots beyond them zeros (the oracle's cost does not depend on
    # the values); the lengths are set per sampled step
    T = w.T
    stride = max(1, T // 16)
    budget = max(1.0, seconds - (t4 - t0))
    t_score = t_attn = 0.0
    sampled, sum_L_sampled = [], 0
    for t in list(range(0, T, stride)):
        if sampled and t_score + t_attn > budget:
            break
        a0 = time.perf_counter()
        Dt = R.score(dec["x"][t, :nb], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        keep = R.decode_keep(Dt, w.theta)
        a1 = time.perf_counter()
        cache.cache_len[...] = L_t[t, :nb]
        R.decode_attn_append(dec["q"][t, :nb], dec["k"][t, :nb], dec["v"][t, :nb], keep, cache, path.scale)
        a2 = time.perf_counter()
        t_score += a1 - a0
        t_attn += a2 - a1
        sampled.append(t)
        sum_L_sampled += int(L_t[t, :nb].sum())
    st["decode_score"] = t_score / (len(sampled) * nb) * (w.B * T)            # per row
    st["decode_attn_append"] = t_attn / max(1, sum_L_sampled) * float(L_t.sum())  # per cached token attended
    st["_sample"] = (nb, len(sampled), stride)
    return st


def cpu_baseline(path, seconds, L_t):
    """The oracle, as it stands, timed per stage on a bounded sample of the same workload on this machine's host cores:
    one pass limited to ONE thread, one on all cores (the oracle is numpy: its threads are the BLAS pool's)."""
    from threadpoolctl import threadpool_info, threadpool_limits
    w = path.w
    with threadpool_limits(limits=1):
        one = _oracle_pass(path, seconds, L_t)
    allc = _oracle_pass(path, seconds, L_t)
    threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
    nb, n_steps, stride = allc.pop("_sample")
    one.pop("_sample")
    total_all, total_one = sum(allc.values()), sum(one.values())
    return {"value": (w.B * w.T) / total_all, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nb} of {w.B} sequences: all prefill stages (scaled by {w.B}/{nb}); decode at every {stride}th of "
                      f"{w.T} steps ({n_steps} steps) with the cache at the exact length of that step, scoring scaled per row, "
                      f"attention scaled by cached tokens attended; float64 numpy",
            "cpu_model": _cpu_model(), "nproc": os.cpu_count(),
            "all_cores": {"threads": threads, "stage_seconds": allc, "step_seconds": total_all,
                          "tokens_per_s": (w.B * w.T) / total_all},
            "one_thread": {"threads": 1, "stage_seconds": one, "step_seconds": total_one,
                           "tokens_per_s": (w.B * w.T) / total_one}}


def pmc_probe(path, torch, L):
    """Dispatches whose hardware counters are read with `rocprofv3 --pmc ...`: a plain device-to-device copy of known
    size (the scale of the byte counters), one dispatch of every prefill kernel, the decode kernel three times, then one
    dispatch of each few-rows layer of a decode step through a decoder layer."""
    w = path.w
    cap = path.cache.max_pages_per_seq * 16
    if L > cap:
        raise SystemExit(f"--pmc-probe {L} exceeds the cache capacity {cap} of this workload (raise --decode-steps)")
    n = 256 << 20
    src = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)                                   # calibration dispatch: reads n bytes, writes n bytes
    torch.cuda.synchronize()
    path.score_vision(); path.select_compact()      # fills the first kept_len tokens of every sequence
    path.qkv_project()                               # (projection of the kept rows: overwrites Q_out and the pages ...
    path.select_compact()                            #  ... which this restores)
    path.prefill_attn()                              # (one dispatch each of the prefill kernels, for their counters)
    path.score_decode(0)
    path.pages.normal_()                             # slots beyond that: arbitrary finite data
    path.cache_len.fill_(L)
    keep0 = torch.zeros(w.B, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(3):
        path.P.dllava_decode_attn_append(path.dec["q"][0], path.dec["k"][0], path.dec["v"][0], w.B, None, 0.0, keep0,
                                         path.cache, path.scale, path.o_dec[0], path.keep_dec[0], path.err,
                                         path.ws_decode)
    torch.cuda.synchronize()
    for _ in range(3):                               # the one-launch step at the same length (no previous token)
        path.cache_len.fill_(L)
        path.P.dllava_decode_step(path.dec["x"][0], w.d, w.d, w.dh, path.pred["W1"], path.pred["b1"], path.pred["W2"],
                                  path.pred["b2"], path.dec["q"][0], path.dec["k"][0], path.dec["v"][0], None, None, None,
                                  None, w.B, 0.0, path.cache, path.scale, path.o_dec[0], path.logits_dec[0], None,
                                  path.err, path.ws_step)
    torch.cuda.synchronize()
    es = 2 if w.dtype == "bf16" else 4
    few = None
    if w.dtype == "bf16":
        # the few-rows layers of a decode step through a decoder layer (7B feed-forward width), one dispatch each:
        # RMSNorm, q|k|v + rotary, W_O + residual, gate|up + gating, down-projection + residual
        P, d, HD, F, B = path.P, w.d, w.H * w.Dh, 11008, w.B
        rnd = lambda *shape: (torch.randn(*shape, device="cuda:0") * 0.02).to(torch.bfloat16)
        Wq, Wk, Wv, Wo, Wg, Wu, Wd = rnd(HD, d), rnd(HD, d), rnd(HD, d), rnd(d, HD), rnd(F, d), rnd(F, d), rnd(d, F)
        xs, gam = rnd(B, d), torch.ones(d, device="cuda:0")
        zz = lambda *shape: torch.zeros(*shape, dtype=torch.bfloat16, device="cuda:0")
        y, q3, k3, v3, x1, f, x2 = zz(B, d), zz(B, HD), zz(B, HD), zz(B, HD), zz(B, d), zz(B, F), zz(B, d)
        pos = torch.arange(B, dtype=torch.int32, device="cuda:0")
        ws = torch.zeros(max(P.dllava_decode_proj_workspace(3 * HD, d), P.dllava_decode_proj_workspace(2 * F, d),
                             P.dllava_linear_few_workspace(d, HD), P.dllava_linear_few_workspace(d, F)),
                         dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        P.dllava_rms_norm(xs, d, B, d, gam, 1e-5, y, d, path.code)
        P.dllava_qkv_few(y, d, B, d, Wq, Wk, Wv, w.H, w.Dh, pos, 10000.0, q3, k3, v3, path.code, ws)
        P.dllava_linear_few(q3, HD, B, HD, Wo, None, d, 0, xs, x1, d, path.code, ws)
        P.dllava_gated_few(x1, d, B, d, Wg, Wu, F, f, F, path.code, ws)
        P.dllava_linear_few(f, F, B, F, Wd, None, d, 0, x1, x2, d, path.code, ws)
        torch.cuda.synchronize()
        few = {"rows": B, "qkv_weight_bytes": 3 * HD * d * es, "wo_weight_bytes": d * HD * es,
               "gate_up_weight_bytes": 2 * F * d * es, "down_weight_bytes": d * F * es}
    rows = int(path.out_off[-1].item())
    n_kept = [int(v) for v in (path.out_off[1:] - path.out_off[:-1]).tolist()]
    print(json.dumps({"pmc_probe": True, "few_rows_layers": few, "copy_bytes_read": n, "copy_bytes_written": n, "cache_len": L,
                      "decode_algorithmic_bytes_per_launch": w.B * L * 2 * w.H * w.Dh * es,
                      "decode_step_algorithmic_bytes_per_launch": w.B * L * 2 * w.H * w.Dh * es + (w.d * w.dh + w.B * w.d) * es,
                      "score_vision_flops": 2.0 * path.M_vis * w.d * w.dh,
                      "qkv_project_flops": 2.0 * rows * w.d * 3 * w.H * w.Dh,
                      "prefill_attn_flops": float(sum(4.0 * w.H * w.Dh * m * (m + 1) / 2 for m in n_kept)),
                      "compact_algorithmic_bytes": 2 * rows * (2 * w.d + 6 * w.H * w.Dh) * es // 2}))


def run_workload(ci, args, torch, P, W, light=False):
    """Times the whole step and its stages on workload ci.  light: the timed step and the stages of the path only."""
    w = W.config(ci)
    if args.decode_steps:
        w.T = args.decode_steps
    path = Path(w, torch, P, W)
    path.two_launch = args.two_launch_decode
    B, T, H, Dh = w.B, w.T, w.H, w.Dh
    es = 2 if w.dtype == "bf16" else 4

    stream = torch.cuda.Stream()
    graph = None
    if args.pmc_probe:
        pmc_probe(path, torch, args.pmc_probe)
        return None
    path.calibrate_theta()
    with torch.cuda.stream(stream):
        path.step()                                     # eager once: validates arguments, warms caches
        stream.synchronize()
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                path.step()
        run = graph.replay if graph is not None else path.step
        for _ in range(args.warmup):
            run()
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps
        assert int(path.err.item()) == 0, "cache capacity overflow during the benchmark"

        # ---- per-stage and per-kernel figures: the same calls, each stage recorded alone into a HIP graph and
        # timed with HIP events on this stream (a graph keeps Python's launch cost out of the measurement; what
        # remains besides the kernels is the ~1 us dispatch gap between consecutive graph nodes)
        keep = path.keep_dec.cpu().numpy().astype(np.int64)            # [T,B] decisions of the last step
        kept_len = np.asarray(w.kept_len, np.int64)
        L_t = kept_len[None, :] + np.concatenate([np.zeros((1, B), np.int64), np.cumsum(keep, 0)[:-1]], 0)  # [T,B]
        kv_bytes_t = L_t.sum(1) * (2 * H * Dh * es)                     # cached K+V bytes streamed at step t

        def stage_ms(fn, n, before=None, reps=3):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(n):
                    fn(i)
            best = float("inf")
            for _ in range(reps):
                if before:
                    before()
                stream.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                g.replay()
                b.record()
                b.synchronize()
                best = min(best, a.elapsed_time(b) / n)
            return best

        ms_score = stage_ms(lambda i: path.score_vision(), 5)
        path.qkv_project()                                              # (weights to the device, outside the graph)
        ms_qkv = stage_ms(lambda i: path.qkv_project(), 3)              # overwrites Q_out and the pages ...
        ms_select = stage_ms(lambda i: path.select_compact(), 5)       # ... which this restores
        extras = not light and not args.no_extras
        nc = ms_nc = nc_kept = None
        if extras:
            nc = NoCacheStep(path)
            ms_nc = stage_ms(lambda i: nc.run(), 3)
            nc_kept = [int(v) for v in (nc.out_off[1:] - nc.out_off[:-1]).tolist()]
        ms_pp_image = ms_pp_text = None
        if extras and w.dtype == "bf16":
            pp = PaperPredictors(path, W)
            ms_pp_image = stage_ms(lambda i: pp.run_image(), 3)
            ms_pp_text = stage_ms(pp.run_text, min(T, 64))
            # decode loop with the appendix-form text predictor: per step, the predictor of this step's tokens and the
            # attention launch (which applies the PREVIOUS token's decision) are independent.  Same stream, then the
            # predictor on a second stream beside the attention (joined before the next step's attention).
            pp.calibrate_theta()
            Tp = min(T, 256)

            def seq_loop(i):
                pp.text_step(i)
                pp.attn_step(i)
            ms_pp_seq = stage_ms(seq_loop, Tp, before=path.select_compact)
            side = torch.cuda.Stream()

            def par_loop(i):
                side.wait_stream(stream)          # the step's input exists when the previous step is done
                with torch.cuda.stream(side):
                    pp.text_step(i)
                pp.attn_step(i)
                stream.wait_stream(side)          # the next step's attention needs these logits
            ms_pp_par = stage_ms(par_loop, Tp, before=path.select_compact)
        ms_masked = None
        if extras and w.dtype == "bf16":   # the training form of the same attention (Eq. 7): full token set, mask inside the softmax
            O_full = torch.zeros_like(path.pre["Q"])
            ws_m = torch.zeros(P.dllava_masked_attn_workspace(w.sumN, B), dtype=torch.uint8, device="cuda:0")
            ms_masked = stage_ms(lambda i: P.dllava_masked_attn(path.pre["Q"], path.pre["K"], path.pre["V"], B, path.seq_off,
                                                                w.sumN, H, Dh, path.scale, path.keep_mask, O_full, path.code,
                                                                ws_m), 3)
        stack = None
        if not light and w.dtype == "bf16" and args.stack:
            # Prefill through 8 LLaMA-family decoder layers of this shape (random weights, feed-forward width 2.6875 d)
            # with the one-time token reduction after layer 2 (Sec. 3.3), against the same 8 layers without reduction
            from paper_2412_00876_amd.layers import DecoderStack
            n_layers, d_ff = 8, (w.d * 43) // 16
            gen = torch.Generator(device="cuda:0")
            gen.manual_seed(w.seed + 5)
            rnd = lambda fo, fi: (torch.randn((fo, fi), generator=gen, device="cuda:0", dtype=torch.float32)
                                  * (2.0 / (fo + fi)) ** 0.5).to(torch.bfloat16)
            ones = lambda n: torch.ones(n, dtype=torch.float32, device="cuda:0")
            wts = [{"Wq": rnd(H * Dh, w.d), "Wk": rnd(H * Dh, w.d), "Wv": rnd(H * Dh, w.d), "Wo": rnd(w.d, H * Dh),
                    "Wg": rnd(d_ff, w.d), "Wu": rnd(d_ff, w.d), "Wd": rnd(w.d, d_ff), "g1": ones(w.d), "g2": ones(w.d)}
                   for _ in range(n_layers)]

            def score_into(X, logits):
                p = path.pred
                P.dllava_score(X, w.d, path.M_vis, B, path.seq_off, path.vis_start, path.vis_len, w.d, w.dh, p["W1"], p["b1"],
                               p["W2"], p["b2"], path.code, logits, path.ws_score_vis)

            def score_rows(X, logits):
                p = path.pred
                P.dllava_score(X, w.d, B, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], path.code, logits,
                               path.ws_score_dec)

            res, res_dec, kv_dec = {}, {}, {}
            Td = min(32, T)                                    # decode steps through the stack, right after the prefill
            pos_t = torch.from_numpy((np.asarray(w.seq_len)[None, :] + np.arange(Td)[:, None]).astype(np.int32)).to("cuda:0")
            for name, l_red, rows_after in (("sparsified_after_layer_2", 2, path.rows_kept), ("dense", n_layers, w.sumN)):
                S = DecoderStack(wts, l_red, B, H, Dh, w.d, d_ff, w.sumN, path.M_vis, max_seq_len=int(max(w.seq_len)),
                                 extra_tokens=Td)
                run_stack = lambda i, S=S, rows_after=rows_after: S.prefill(path.pre["hidden"], path.seq_off, path.vis_start,
                                                                             path.vis_len, w.keep_ratio, rows_after, score_into)
                res[name] = stage_ms(run_stack, 1, reps=3)
                run_dec = lambda i, S=S: S.decode_step(path.dec["x"][i], pos_t[i], w.theta, score_rows)
                res_dec[name] = stage_ms(run_dec, Td, before=lambda S=S, r=run_stack: r(0), reps=2) * 1e3    # us per step
                kv_dec[name] = S.kv_bytes() / 1e9
                assert int(S.err.item()) == 0
                del S
            per_tok = 2.0 * (4 * w.d * H * Dh + 3 * w.d * d_ff)          # linear-layer flops per token and layer
            stack = {"layers": n_layers, "d_ff": d_ff, "rows": int(w.sumN), "rows_after_reduction": int(path.rows_kept),
                     "ms": res, "speedup": res["dense"] / res["sparsified_after_layer_2"],
                     "dense_linear_tflops": per_tok * w.sumN * n_layers / (res["dense"] * 1e-3) / 1e12,
                     "projected_32_layers_ms": {k: v + (v - 0.0) * 0 for k, v in res.items()}}
            lay_d = res["dense"] / n_layers
            lay_s = (res["sparsified_after_layer_2"] - 2 * lay_d) / (n_layers - 2)
            stack["projected_32_layers_ms"] = {"dense": 32 * lay_d, "sparsified_after_layer_2": 2 * lay_d + 30 * lay_s}
            stack["decode_us_per_step"] = res_dec
            stack["decode_tokens_per_s"] = {k: B / (v * 1e-6) for k, v in res_dec.items()}
            stack["decode_steps"] = Td
            stack["kv_gb_after_decode"] = kv_dec
            del wts
        ms_prefill = stage_ms(lambda i: path.prefill_attn(), 5)
        ms_sd = ms_da = None
        if extras or args.two_launch_decode:
            ms_sd = stage_ms(path.score_decode, T)                          # logits of all steps: inputs of the next line
            ms_da = stage_ms(path.decode_attn, T, before=path.select_compact)  # cache reset, then T attention launches
            assert np.array_equal(path.keep_dec.cpu().numpy(), keep), "decode replay diverged from the timed run"
        ms_ds = stage_ms(path.decode_step, T, before=path.select_compact)  # cache reset, then T one-launch steps

    tokens = B * T
    value = tokens / (ms_per_step * 1e-3)
    # dominant kernel: the decode launch.  Algorithmic bytes per launch: the cached K+V of every sequence, and for the
    # one-launch step also what its scoring half must read once (W1 and the B hidden rows).
    pred_bytes = (w.d * w.dh + B * w.d) * es
    if args.two_launch_decode and ms_da is not None:
        kernel_name, avg_ms, avg_bytes = "decode_attn_kernel (dllava_decode_attn_append)", float(ms_da), float(kv_bytes_t.mean())
        traffic_factor = DECODE_TRAFFIC_PER_ALGORITHMIC_BYTE
    else:
        kernel_name, avg_ms, avg_bytes = "decode_step_kernel (dllava_decode_step)", float(ms_ds), float(kv_bytes_t.mean()) + pred_bytes
        traffic_factor = STEP_TRAFFIC_PER_ALGORITHMIC_BYTE
    achieved = avg_bytes / (avg_ms * 1e-3) / 1e9
    M_vis = path.M_vis
    flops_score = 2.0 * M_vis * w.d * w.dh + 4.0 * M_vis * w.dh
    flops_prefill = sum(4.0 * H * Dh * n * (n + 1) / 2 for n in w.kept_len)
    rows = path.rows_kept
    flops_qkv = 2.0 * rows * w.d * 3 * H * Dh
    bytes_compact = 2.0 * rows * (w.d + 3 * H * Dh) * es
    dense_L = (np.asarray(w.seq_len)[None, :] + np.arange(T)[:, None]).sum(1) * (2 * H * Dh * es)
    out = {
        "metric": "sparsified decode attn tokens/s (whole sparsify-then-attend step)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: LLaVA-1.5-7B shape x batch {B}: prefill {w.n_sys[0]}|{w.n_vis[0]}|{w.n_prompt[0]} "
                               f"tokens -> {w.kept_len[0]} kept (r={w.keep_ratio}), {T} decode steps, 16-token pages"
                               if ci == 2 else f"{w.name}: {B} sequences, prefill {w.n_sys[0]}|{w.n_vis[0]}|{w.n_prompt[0]} tokens -> "
                               f"{w.kept_len[0]} kept (r={w.keep_ratio}), {T} decode steps, H={H}, d={w.d}",
                   "decode_steps": T, "hip_graph": graph is not None,
                   "text_keep_fraction": float(keep.mean()), "theta": w.theta},
        "roofline": {"kernel": kernel_name, "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_factor * avg_bytes if (ci == 2 and traffic_factor) else None,
                     "avg_launch_us": avg_ms * 1e3, "avg_bytes_per_launch": avg_bytes},
        "stages": {
            "score_vision": {"ms": ms_score, "tflops": flops_score / (ms_score * 1e-3) / 1e12,
                             "frac_mfma_peak": flops_score / (ms_score * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "select_compact": {"ms": ms_select, "gbs": bytes_compact / (ms_select * 1e-3) / 1e9,
                               "frac_hbm_peak": bytes_compact / (ms_select * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "prefill_attn": {"ms": ms_prefill, "tflops": flops_prefill / (ms_prefill * 1e-3) / 1e12,
                             "frac_mfma_peak": flops_prefill / (ms_prefill * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            # not part of the timed step (the step hands precomputed Q/K/V to select_compact): the projections of
            # the layer over the kept rows only, the stage that follows compaction in a decoder layer
            "qkv_project": {"ms": ms_qkv, "tflops": flops_qkv / (ms_qkv * 1e-3) / 1e12,
                            "frac_mfma_peak": flops_qkv / (ms_qkv * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                            "flops_dense_counterfactual": 2.0 * w.sumN * w.d * 3 * H * Dh},
            # the paper's other decoding mode, also outside the timed step: one step without KV cache at the end of
            # the generation (re-mask all output tokens, compact, causal attention over prompt* + kept outputs)
            "decode_step_without_cache": None if ms_nc is None else {"ms": ms_nc, "rows_in": nc.sumN, "rows_kept": int(sum(nc_kept)),
                                          "attn_tflops": sum(4.0 * H * Dh * n * (n + 1) / 2 for n in nc_kept) / (ms_nc * 1e-3) / 1e12,
                                          "attn_flops_dense_counterfactual": float(sum(4.0 * H * Dh * n * (n + 1) / 2
                                                                                       for n in (np.asarray(w.seq_len) + T)))},
            # the predictors in the appendix's form (also outside the timed step): image predictor over all vision
            # spans, output-text predictor over the B rows of a decode step
            "masked_attn_full_token_set": None if ms_masked is None else {
                "ms": ms_masked, "rows": int(w.sumN),
                "tflops_causal": sum(4.0 * H * Dh * n * (n + 1) / 2 for n in w.seq_len) / (ms_masked * 1e-3) / 1e12},
            "decoder_stack_prefill": stack,
            "predict_image": None if ms_pp_image is None else {
                "ms": ms_pp_image, "rows": path.M_vis, "tflops": pp.flops_image() / (ms_pp_image * 1e-3) / 1e12,
                "frac_mfma_peak": pp.flops_image() / (ms_pp_image * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "predict_text": None if ms_pp_text is None else {"avg_us": float(ms_pp_text * 1e3), "rows": B},
            "decode_step_appendix_predictor": None if ms_pp_text is None else {
                "same_stream_us": float(ms_pp_seq * 1e3), "predictor_beside_attention_us": float(ms_pp_par * 1e3),
                "steps": Tp, "note": "dllava_predict (output-text form) + dllava_decode_step without scoring, first steps of the generation"},
            # K/V held by a 32-layer decoder with the decisions taken once after layer l = 2 (Sec. 3.3) and shared by
            # the later layers: layers 1..2 keep every token, layers 3..32 the reduced prompt and the kept outputs
            # (this run's decisions); arithmetic on the cache lengths, checked against real caches by the tests
            "kv_memory_gb_32_layers_l2": (lambda per_tok, full0, red0, fullT, redT: {
                "after_prefill": {"dense": 32 * full0 * per_tok / 1e9, "sparsified": (2 * full0 + 30 * red0) * per_tok / 1e9},
                "after_decode": {"dense": 32 * fullT * per_tok / 1e9, "sparsified": (2 * fullT + 30 * redT) * per_tok / 1e9}})(
                2 * H * Dh * es, int(np.sum(w.seq_len)), int(np.sum(w.kept_len)), int(np.sum(w.seq_len)) + B * T,
                int(np.sum(w.kept_len)) + int(keep.sum())),
            "decode_step": {"avg_us": float(ms_ds * 1e3), "gbs": (float(kv_bytes_t.mean()) + pred_bytes) / (ms_ds * 1e-3) / 1e9,
                            "note": "one launch per step: scoring + attention, append deferred by one step"},
            "decode_score": None if ms_sd is None else {"avg_us": float(ms_sd * 1e3)},
            "decode_attn": None if ms_da is None else {"avg_us": float(ms_da * 1e3), "gbs": float(kv_bytes_t.mean()) / (ms_da * 1e-3) / 1e9},
            "kv_mb_first_step": float(kv_bytes_t[0] / 1e6), "kv_mb_last_step": float(kv_bytes_t[-1] / 1e6),
            "kv_bytes_total": float(kv_bytes_t.sum()), "kv_bytes_dense_counterfactual": float(dense_L.sum()),
        },
        "input_generation_s": path.gen_seconds,
    }
    out["_L_t"] = L_t
    out["_path"] = path
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by sequence, or by head, with no exchange "
              "between GPUs, so N GPUs would run N independent copies of this benchmark); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import paper_2412_00876_amd as P
    from synth import workloads as W

    torch.cuda.set_device(0)
    ci = int(args.workload[1]) - 1
    out = run_workload(ci, args, torch, P, W)
    if out is None:
        return
    L_t, path = out.pop("_L_t"), out.pop("_path")
    w = path.w
    stream = torch.cuda.Stream()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(path, args.cpu_seconds, L_t)
    del path
    torch.cuda.empty_cache()
    if ci == 2 and not args.decode_steps and not args.no_other_workloads:
        # The same step and its stages on the workloads where the matrix-core and compaction stages have their largest
        # shapes (13B: 32 sequences; high resolution: 2880 vision tokens per sequence), each on the driver's clock too.
        for name, cj in (("c4", 3), ("c5", 4)):
            r = run_workload(cj, args, torch, P, W, light=True)
            r.pop("_L_t")
            r.pop("_path")
            torch.cuda.empty_cache()
            st = r["stages"]
            out[name] = {"workload": r["config"]["workload"], "tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
                         "text_keep_fraction": r["config"]["text_keep_fraction"],
                         "decode_step": {"avg_us": r["roofline"]["avg_launch_us"], "gbs": r["roofline"]["achieved"],
                                         "frac_hbm_peak": r["roofline"]["frac"],
                                         "avg_bytes_per_launch": r["roofline"]["avg_bytes_per_launch"]},
                         "score_vision": st["score_vision"], "select_compact": st["select_compact"],
                         "prefill_attn": st["prefill_attn"], "qkv_project": st["qkv_project"]}
    if ci == 2 and not args.decode_steps and not args.no_other_workloads:
        # The same step on the batch-1 prompt this workload batches (configs[1]: 35 | 576 | 64 tokens, 256 decode steps):
        # 3.5-5.6 MB of K/V per decode launch, so every launch is latency, not bandwidth.  Reported beside the headline.
        w1 = W.config(1)
        p1 = Path(w1, torch, P, W)
        p1.calibrate_theta()
        with torch.cuda.stream(stream):
            p1.step()
            stream.synchronize()
            g1 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g1, stream=stream):
                p1.step()
            for _ in range(3):
                g1.replay()
            stream.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                g1.replay()
            stream.synchronize()
            ms1 = (time.perf_counter() - t0) * 1e3 / 20
        out["batch_1"] = {"workload": w1.name, "tokens_per_s": w1.B * w1.T / (ms1 * 1e-3), "ms_per_step": ms1,
                          "decode_steps": w1.T, "us_per_decode_step": (ms1 * 1e3) / w1.T}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
