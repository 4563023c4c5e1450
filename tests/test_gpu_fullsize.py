"""GPU parity at the benchmark's full shapes (C3, C4, C5), in the launch configurations bench.py times.

The oracle cannot run these sizes whole in seconds, so integer work is still compared in full (it is cheap on the
CPU) while floating outputs are compared on sampled rows / (sequence, head) pairs that the oracle computes one by one.
Decode runs a bounded number of steps from the compacted prefill cache, plus one step on a long, host-filled cache
at the context length the configuration reaches at its end."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_parity import TOL, _assert_out_close

STEPS = 24


def _H():
    from tests import harness
    return harness


def _sample(rs, n, k):
    return sorted(set(int(x) for x in rs.choice(n, size=min(k, n), replace=False)))


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_full_shape_path(ci):
    h = _H()
    w = W.config(ci)
    w.T = STEPS
    rs = np.random.RandomState(100 + ci)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w)
    g = h.GpuPath(w, pre, pred)

    # ---- scoring: all vision rows on the GPU, sampled rows in the oracle
    D = g.score_vision()
    D_np = D.cpu().numpy()
    assert np.isfinite(D_np).all()
    vis_rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                               for b in range(w.B)])
    pick = _sample(rs, len(vis_rows), 96) + [0, len(vis_rows) - 1]
    ref = R.score(pre["hidden"][vis_rows[pick]], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    assert np.abs(D_np[pick] - ref).max() <= TOL

    # ---- selection + compaction on the GPU's own logits: bit-exact, in full
    out = g.select_compact(D)
    mask, idx, off = R.select(D_np, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    total = int(off[-1])
    assert total == sum(w.kept_len)
    assert np.array_equal(out["out_off"].cpu().numpy(), off)
    assert np.array_equal(out["keep_mask"].cpu().numpy(), mask)
    assert np.array_equal(out["kept_idx"].cpu().numpy()[:total], idx)
    assert np.array_equal(g.cache_len.cpu().numpy(), np.diff(off))
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)])
    assert np.array_equal(h.bits(out["hidden_out"])[:total], pre["hidden"][src])
    assert np.array_equal(h.bits(out["Q_out"])[:total], pre["Q"][src])
    cache = R.PagedCache(g.pages.shape[0], g.bt_np, w.H, w.Dh, w.dtype)
    R.compact(idx, off, w.seq_off, K=pre["K"], V=pre["V"], cache=cache)
    assert np.array_equal(h.bits(g.pages), cache.pages)

    # ---- prefill attention from the pages: sampled (sequence, head), a spread of rows each
    O = g.prefill(out["Q_out"][:total].contiguous(), out["out_off"])
    Oh = h.as_f64(O)
    Qc, Kc, Vc = pre["Q"][src], pre["K"][src], pre["V"][src]
    for _ in range(6):
        b, hd = int(rs.randint(w.B)), int(rs.randint(w.H))
        r0, r1 = int(off[b]), int(off[b + 1])
        o_ref = R.prefill_attn(Qc[r0:r1, hd:hd + 1], Kc[r0:r1, hd:hd + 1], Vc[r0:r1, hd:hd + 1],
                               np.array([0, r1 - r0]), g.scale, w.dtype)
        _assert_out_close(Oh[r0:r1, hd:hd + 1], o_ref, w.dtype, f"prefill b={b} h={hd}")

    # ---- decode: STEPS steps with GPU scores; decisions taken from the GPU logits on both sides
    pairs = [(int(rs.randint(w.B)), int(rs.randint(w.H))) for _ in range(6)] + [(0, 0), (w.B - 1, w.H - 1)]
    for t in range(w.T):
        x = h.to_dev(dec["x"][t], w.dtype)
        Dg = g.score_rows(x)
        Dg_np = Dg.cpu().numpy()
        Dr = R.score(dec["x"][t], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        assert np.abs(Dg_np - Dr).max() <= TOL
        keep_ref = R.decode_keep(Dg_np, w.theta)
        q, k, v = (h.to_dev(dec[n][t], w.dtype) for n in ("q", "k", "v"))
        o, keep = g.decode(q, k, v, logits=Dg, theta=w.theta)
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep_ref, cache, g.scale, only=pairs)
        assert not err.any()
        assert np.array_equal(keep.cpu().numpy(), keep_ref)
        assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
        oh = h.as_f64(o)
        for b, hd in pairs:
            _assert_out_close(oh[b, hd], o_ref[b, hd], w.dtype, f"decode t={t} b={b} h={hd}")
    assert int(g.err.item()) == 0
    assert np.array_equal(h.bits(g.pages), cache.pages)


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_decode_step_at_final_context_length(ci):
    """One decode step per configuration at the cache length it reaches at the end of its run (ragged by a few tokens
    per sequence), on a cache whose pages were filled on the host."""
    h = _H()
    w = W.config(ci)
    rs = np.random.RandomState(200 + ci)
    L_end = w.kept_len[0] + w.T // 2
    lens = np.array([L_end - int(rs.randint(0, 40)) for _ in range(w.B)], np.int32)
    bt, n_pages = W.block_table(w)
    g = h.GpuPath(w, None, None, n_pages=n_pages, bt=bt)
    pages_np = W.store(rng.normal(w.seed, "final.pages", (n_pages, 2, w.H, 16, w.Dh)), w.dtype)
    g.pages.copy_(h.to_dev(pages_np, w.dtype))
    g.cache_len.copy_(torch.from_numpy(lens))
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    cache.pages[...] = pages_np
    cache.cache_len[...] = lens
    dec = W.decode_inputs(w, 1)
    keep = rng.bernoulli(w.seed, "final.keep", (w.B,), 0.5)
    q, k, v = (h.to_dev(dec[n][0], w.dtype) for n in ("q", "k", "v"))
    o, keep_out = g.decode(q, k, v, keep_override=torch.from_numpy(keep).to(h.DEV))
    pairs = [(int(rs.randint(w.B)), int(rs.randint(w.H))) for _ in range(10)] + [(0, 0), (w.B - 1, w.H - 1)]
    o_ref, err = R.decode_attn_append(dec["q"][0], dec["k"][0], dec["v"][0], keep, cache, g.scale, only=pairs)
    assert not err.any() and int(g.err.item()) == 0
    assert np.array_equal(keep_out.cpu().numpy(), keep)
    assert np.array_equal(g.cache_len.cpu().numpy(), lens + keep)
    oh = h.as_f64(o)
    for b, hd in pairs:
        _assert_out_close(oh[b, hd], o_ref[b, hd], w.dtype, f"b={b} h={hd}")
    assert np.array_equal(h.bits(g.pages), cache.pages)


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_deferred_decode_steps_at_final_context_length(ci):
    """dllava_decode_step in the benchmark's launch configuration (scoring blocks + attention blocks in one launch), at
    the cache length the configuration reaches at its end: three steps and the final commit, outputs of sampled
    (sequence, head) pairs and all logits against the oracle's plain Eq. 6 loop, the cache bit for bit."""
    import paper_2412_00876_amd as P
    h = _H()
    w = W.config(ci)
    rs = np.random.RandomState(300 + ci)
    T = 3
    L_end = w.kept_len[0] + w.T // 2
    lens = np.array([L_end - int(rs.randint(0, 40)) for _ in range(w.B)], np.int32)
    bt, n_pages = W.block_table(w)
    pred = W.predictor(w)
    g = h.GpuPath(w, None, pred, n_pages=n_pages, bt=bt)
    pages_np = W.store(rng.normal(w.seed, "final.pages", (n_pages, 2, w.H, 16, w.Dh)), w.dtype)
    g.pages.copy_(h.to_dev(pages_np, w.dtype))
    g.cache_len.copy_(torch.from_numpy(lens))
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    cache.pages[...] = pages_np
    cache.cache_len[...] = lens
    dec = W.decode_inputs(w, T)
    dev = {n: h.to_dev(dec[n], w.dtype) for n in ("x", "q", "k", "v")}
    ws = torch.zeros(P.dllava_decode_step_workspace(w.B, w.H, w.Dh, g.cache.max_pages_per_seq, w.d, w.dh, g.code),
                     dtype=torch.uint8, device=h.DEV)
    logits = torch.zeros((T, w.B, 2), dtype=torch.float32, device=h.DEV)
    keep_out = torch.full((T, w.B), 255, dtype=torch.uint8, device=h.DEV)
    pairs = [(int(rs.randint(w.B)), int(rs.randint(w.H))) for _ in range(8)] + [(0, 0), (w.B - 1, w.H - 1)]
    p = g.pred
    theta = 0.0
    for t in range(T):
        o = torch.zeros((w.B, w.H, w.Dh), dtype=h.tdtype(w.dtype), device=h.DEV)
        prev = t > 0
        P.dllava_decode_step(dev["x"][t], w.d, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], dev["q"][t], dev["k"][t],
                             dev["v"][t], dev["k"][t - 1] if prev else None, dev["v"][t - 1] if prev else None,
                             logits[t - 1] if prev else None, None, w.B, theta, g.cache, g.scale, o, logits[t],
                             keep_out[t - 1] if prev else None, g.err, ws)
        Dg = logits[t].cpu().numpy()
        Dr = R.score(dec["x"][t], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        assert np.abs(Dg - Dr).max() <= TOL
        keep_ref = R.decode_keep(Dg, theta)          # decisions from the GPU's logits on both sides
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep_ref, cache, g.scale, only=pairs)
        assert not err.any()
        oh = h.as_f64(o)
        for b, hd in pairs:
            _assert_out_close(oh[b, hd], o_ref[b, hd], w.dtype, f"deferred t={t} b={b} h={hd}")
        if prev:
            assert np.array_equal(keep_out[t - 1].cpu().numpy(), R.decode_keep(logits[t - 1].cpu().numpy(), theta))
    P.dllava_decode_commit(dev["k"][T - 1], dev["v"][T - 1], logits[T - 1], None, w.B, theta, g.cache, keep_out[T - 1], g.err)
    assert int(g.err.item()) == 0
    assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
    assert np.array_equal(h.bits(g.pages), cache.pages)
