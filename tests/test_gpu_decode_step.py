"""GPU parity of the deferred decode step (dllava_decode_step + dllava_decode_commit) against the oracle's Eq. 6
loop: the attention outputs must be those of the plain step at every step, the keep decisions arrive one call
later, and after the final commit the cache equals the oracle's bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_parity import TOL, _assert_out_close


def _H():
    from tests import harness
    return harness


def _run(w, T, theta, use_override, extra_tokens=None):
    h = _H()
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w, T), W.predictor(w)
    g = h.GpuPath(w, pre, pred, extra_tokens=T if extra_tokens is None else extra_tokens)
    # prefill state: everything kept text (no vision span in these workloads) -> compacted cache on both sides
    D0 = np.zeros((max(1, int(sum(w.n_vis))), 2), np.float32)   # no vision rows: one unused row keeps the pointer valid
    out = g.select_compact(torch.from_numpy(D0).to(h.DEV), with_hidden=False)
    mask, idx, off = R.select(D0, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    cache = R.PagedCache(g.pages.shape[0], g.bt_np, w.H, w.Dh, w.dtype)
    R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    assert np.array_equal(h.bits(g.pages), cache.pages)

    ws = torch.zeros(P.dllava_decode_step_workspace(w.B, w.H, w.Dh, g.cache.max_pages_per_seq, w.d, w.dh, g.code),
                     dtype=torch.uint8, device=h.DEV)
    td = h.tdtype(w.dtype)
    logits = torch.zeros((T, w.B, 2), dtype=torch.float32, device=h.DEV)
    keep_prev = torch.full((T + 1, w.B), 255, dtype=torch.uint8, device=h.DEV)
    pattern = W.keep_pattern(w, T)
    dev = {n: h.to_dev(dec[n], w.dtype) for n in ("x", "q", "k", "v")}
    p = g.pred
    keeps_ref = []
    for t in range(T):
        o = torch.zeros((w.B, w.H, w.Dh), dtype=td, device=h.DEV)
        prev = t > 0
        ov = torch.from_numpy(pattern[t - 1]).to(h.DEV) if (use_override and prev) else None
        P.dllava_decode_step(dev["x"][t], w.d, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"],
                             dev["q"][t], dev["k"][t], dev["v"][t],
                             dev["k"][t - 1] if prev else None, dev["v"][t - 1] if prev else None,
                             logits[t - 1] if (prev and not use_override) else None, ov,
                             w.B, theta, g.cache, g.scale, o, logits[t], keep_prev[t], g.err, ws)
        # oracle: the plain step of Eq. 6 with the decision taken on the oracle's own logits
        Dr = R.score(dec["x"][t], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        assert np.abs(logits[t].cpu().numpy() - Dr).max() <= TOL
        keep_ref = pattern[t] if use_override else R.decode_keep(Dr, theta)
        if not use_override:   # the two sides decide on their own logits: stay away from ties
            assert np.abs((Dr[:, 1] - Dr[:, 0]) - theta).min() > 10 * np.abs(logits[t].cpu().numpy() - Dr).max()
        lens_before = cache.cache_len.copy()
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep_ref, cache, g.scale)
        assert not err.any()
        _assert_out_close(h.as_f64(o), o_ref, w.dtype, f"step {t}")
        # the GPU cache lags by the token of this step
        assert np.array_equal(g.cache_len.cpu().numpy(), lens_before)
        if prev:
            assert np.array_equal(keep_prev[t].cpu().numpy(), keeps_ref[-1])
        keeps_ref.append(np.asarray(keep_ref, np.uint8))
    ov = torch.from_numpy(pattern[T - 1]).to(h.DEV) if use_override else None
    P.dllava_decode_commit(dev["k"][T - 1], dev["v"][T - 1], None if use_override else logits[T - 1], ov, w.B, theta,
                           g.cache, keep_prev[T], g.err)
    assert np.array_equal(keep_prev[T].cpu().numpy(), keeps_ref[-1])
    assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
    assert np.array_equal(h.bits(g.pages), cache.pages)
    assert int(g.err.item()) == 0


@pytest.mark.parametrize("B,H,Dh,d", [(16, 4, 128, 512),     # fused launch, one column tile of tokens
                                      (20, 2, 128, 256),     # two column tiles
                                      (3, 5, 64, 192),       # the smaller head size, odd head count
                                      (40, 2, 128, 256),     # two row groups of scoring blocks (32 + 8 rows)
                                      (64, 1, 128, 128),     # two full row groups
                                      (70, 2, 128, 256)])    # more rows than the fused scoring takes: two launches
def test_deferred_step_matches_eq6_with_forced_decisions(B, H, Dh, d):
    w = W.make("step", "bf16", d, H, Dh, B, [5 + (7 * b) % 40 for b in range(B)], 0, 0, 1.0, 6, project_qkv=True)
    _run(w, 6, 0.0, use_override=True)


def test_deferred_step_decides_on_its_own_logits():
    w = W.make("steplog", "bf16", 512, 4, 128, 8, [3, 17, 0, 33, 16, 15, 64, 1], 0, 0, 1.0, 8, project_qkv=True)
    _run(w, 8, 0.0, use_override=False)


def test_deferred_step_float32():
    w = W.make("stepf32", "f32", 128, 2, 64, 3, [4, 0, 19], 0, 0, 1.0, 5, project_qkv=True)
    _run(w, 5, 0.0, use_override=True)


def test_deferred_step_at_cache_capacity():
    """A kept token that finds its sequence full is neither stored nor attended by later steps, the flag is raised,
    the length stays at the capacity: the same as the plain step."""
    h = _H()
    B, T = 3, 5
    w = W.make("stepcap", "bf16", 256, 2, 128, B, [14, 16, 3], 0, 0, 1.0, T, project_qkv=True)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w, T), W.predictor(w)
    bt = np.array([[2], [0], [1]], np.int32)        # one page = 16 slots per sequence
    g = h.GpuPath(w, pre, pred, n_pages=3, bt=bt)
    D0 = np.zeros((1, 2), np.float32)
    g.select_compact(torch.from_numpy(D0).to(h.DEV), with_hidden=False)
    mask, idx, off = R.select(D0, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    cache = R.PagedCache(3, bt, w.H, w.Dh, w.dtype)
    R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    ws = torch.zeros(P.dllava_decode_step_workspace(B, w.H, w.Dh, 1, w.d, w.dh, g.code), dtype=torch.uint8, device=h.DEV)
    dev = {n: h.to_dev(dec[n], w.dtype) for n in ("x", "q", "k", "v")}
    logits = torch.zeros((T, B, 2), dtype=torch.float32, device=h.DEV)
    ones = torch.ones(B, dtype=torch.uint8, device=h.DEV)     # every token is kept
    p = g.pred
    any_err = False
    for t in range(T):
        o = torch.zeros((B, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
        prev = t > 0
        P.dllava_decode_step(dev["x"][t], w.d, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], dev["q"][t], dev["k"][t],
                             dev["v"][t], dev["k"][t - 1] if prev else None, dev["v"][t - 1] if prev else None, None,
                             ones if prev else None, B, 0.0, g.cache, g.scale, o, logits[t], None, g.err, ws)
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], np.ones(B, np.uint8), cache, g.scale)
        any_err = any_err or bool(err.any())
        _assert_out_close(h.as_f64(o), o_ref, w.dtype, f"step {t}")
    P.dllava_decode_commit(dev["k"][T - 1], dev["v"][T - 1], None, ones, B, 0.0, g.cache, None, g.err)
    assert any_err and int(g.err.item()) == 1
    assert g.cache_len.cpu().numpy().tolist() == [16, 16, 8] and cache.cache_len.tolist() == [16, 16, 8]
    assert np.array_equal(h.bits(g.pages), cache.pages)


def test_deferred_step_with_logits_from_the_appendix_form_predictor():
    """x == NULL: the call scores nothing; the decisions come from dllava_predict (output-text predictor of the
    appendix) issued beside it.  Outputs and the final cache equal Eq. 6 with the oracle predictor's decisions."""
    from oracle import predictor_ref as PR
    from tests.test_gpu_predictor import upload
    h = _H()
    T = 6
    w = W.make("stepp", "bf16", 256, 4, 128, 5, [9, 30, 2, 17, 44], 0, 0, 1.0, T, project_qkv=True, seed=321)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w, T), W.predictor(w)
    g = h.GpuPath(w, pre, pred, extra_tokens=T)
    D0 = np.zeros((1, 2), np.float32)
    g.select_compact(torch.from_numpy(D0).to(h.DEV), with_hidden=False)
    mask, idx, off = R.select(D0, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    cache = R.PagedCache(g.pages.shape[0], g.bt_np, w.H, w.Dh, w.dtype)
    R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    Pw = W.paper_predictor(w, 0)
    desc = upload(h, Pw, w.d)
    ws_p = torch.empty(P.dllava_predict_workspace(w.B, w.B, 0), dtype=torch.uint8, device=h.DEV)
    ws = torch.zeros(P.dllava_decode_workspace(w.B, w.H, w.Dh, g.cache.max_pages_per_seq), dtype=torch.uint8, device=h.DEV)
    logits = torch.zeros((T, w.B, 2), dtype=torch.float32, device=h.DEV)
    dev = {n: h.to_dev(dec[n], w.dtype) for n in ("x", "q", "k", "v")}
    theta = 0.0
    side = torch.cuda.Stream()
    for t in range(T):
        o = torch.zeros((w.B, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
        prev = t > 0
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):      # the predictor of THIS step's tokens, beside the attention launch
            P.dllava_predict(dev["x"][t], w.d, w.B, 0, None, None, None, desc, P.BF16, logits[t], ws_p)
        P.dllava_decode_step(None, 0, 0, 0, None, None, None, None, dev["q"][t], dev["k"][t], dev["v"][t],
                             dev["k"][t - 1] if prev else None, dev["v"][t - 1] if prev else None,
                             logits[t - 1] if prev else None, None, w.B, theta, g.cache, g.scale, o, None, None, g.err, ws)
        torch.cuda.current_stream().wait_stream(side)
        Dr = PR.predict(dec["x"][t], None, Pw, "bf16")
        Dg = logits[t].cpu().numpy()
        assert np.abs(Dg - Dr).max() <= TOL
        assert np.abs((Dr[:, 1] - Dr[:, 0]) - theta).min() > 10 * np.abs(Dg - Dr).max()      # away from ties
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], R.decode_keep(Dr, theta), cache, g.scale)
        assert not err.any()
        _assert_out_close(h.as_f64(o), o_ref, w.dtype, f"step {t}")
    P.dllava_decode_commit(dev["k"][T - 1], dev["v"][T - 1], logits[T - 1], None, w.B, theta, g.cache, None, g.err)
    assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
    assert np.array_equal(h.bits(g.pages), cache.pages)
    assert int(g.err.item()) == 0
