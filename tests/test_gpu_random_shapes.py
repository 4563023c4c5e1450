"""Seeded random shapes through the whole path (every entry point, both decode forms) against the oracle: batch sizes,
head counts, head sizes, hidden sizes, storage types and span layouts the hand-picked cases do not cover."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_parity import TOL, TOL_F32, _assert_out_close


def _H():
    from tests import harness
    return harness


def _random_workload(seed):
    rs = np.random.RandomState(1000 + seed)
    dtype = "f32" if seed % 5 == 4 else "bf16"
    B = int(rs.randint(1, 10))
    H = int(rs.randint(1, 7))
    Dh = int(rs.choice([64, 128]))
    d = int(rs.choice([64, 128, 192, 256, 320]))
    n_sys = [int(rs.randint(0, 6)) for _ in range(B)]
    n_vis = [int(rs.choice([0, 1, 7, 40, 130, 300])) for _ in range(B)]
    n_prompt = [int(rs.randint(0, 20)) for _ in range(B)]
    if sum(n_sys) + sum(n_vis) + sum(n_prompt) == 0:
        n_prompt[0] = 3
    ratio = float(rs.choice([0.0, 0.2, 0.5, 0.93, 1.0]))
    T = int(rs.randint(2, 6))
    return W.make(f"random{seed}", dtype, d, H, Dh, B, n_sys, n_vis, n_prompt, ratio, T, project_qkv=True, seed=7000 + seed)


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_whole_path(seed):
    h = _H()
    w = _random_workload(seed)
    tol = TOL if w.dtype == "bf16" else TOL_F32
    pre, dec, pred, aw = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w), W.attn_weights(w)
    pred["b1"] = rng.normal(w.seed, "b1", (w.dh,)).astype(np.float32) * 0.1      # biases on
    pred["b2"] = rng.normal(w.seed, "b2", (2,)).astype(np.float32) * 0.1
    g = h.GpuPath(w, pre, pred)

    # scoring of the vision spans
    vis = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                          for b in range(w.B)]).astype(np.int64)
    if len(vis):
        D_ref = R.score(pre["hidden"][vis], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        assert np.abs(g.score_vision().cpu().numpy() - D_ref).max() <= tol
    else:
        D_ref = np.zeros((1, 2), np.float32)
    # selection + compaction on identical logits: bit-exact
    out = g.select_compact(torch.from_numpy(D_ref).to(h.DEV))
    mask, idx, off = R.select(D_ref[:len(vis)] if len(vis) else D_ref[:0], w.seq_off, w.vis_start, w.vis_len, R.TOPK,
                              w.keep_ratio, 0.0)
    total = int(off[-1])
    assert np.array_equal(out["keep_mask"].cpu().numpy(), mask)
    assert np.array_equal(out["out_off"].cpu().numpy(), off)
    assert np.array_equal(out["kept_idx"].cpu().numpy()[:total], idx)
    cache = R.PagedCache(g.pages.shape[0], g.bt_np, w.H, w.Dh, w.dtype)
    h_star, Qc = R.compact(idx, off, w.seq_off, hidden=pre["hidden"], Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    assert np.array_equal(h.bits(g.pages), cache.pages)
    assert np.array_equal(h.bits(out["hidden_out"])[:total], h_star)
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)]) if total else np.zeros(0, np.int64)
    # prefill attention from the pages
    if total:
        O = g.prefill(out["Q_out"].contiguous(), out["out_off"])
        O_ref = R.prefill_attn(Qc, pre["K"][src], pre["V"][src], off, g.scale, w.dtype)
        _assert_out_close(h.as_f64(O[:total]), O_ref, w.dtype, "prefill")
        # projection of the compacted hidden states into a second cache
        g2 = h.GpuPath(w, pre, pred)
        Wd = {k: h.to_dev(v, w.dtype) for k, v in aw.items()}
        Q2 = torch.zeros((w.sumN, w.H, w.Dh), dtype=h.tdtype(w.dtype), device=h.DEV)
        P.dllava_qkv_project(out["hidden_out"], w.d, w.sumN, w.d, w.B, out["out_off"], out["kept_idx"], Wd["q"], Wd["k"],
                             Wd["v"], 10000.0, Q2, g2.cache, g2.err, g2.code)
        Qr, Kr, Vr = R.qkv_project(h_star, off, idx[:total], aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, 10000.0)
        _assert_out_close(h.as_f64(Q2[:total]), Qr, w.dtype, "projected Q")
        assert np.array_equal(g2.cache_len.cpu().numpy(), np.diff(off))
        for b in range(w.B):
            n = int(off[b + 1] - off[b])
            if n:
                Kg, Vg = g2.cache_rows(b, n)
                _assert_out_close(R.widen(Kg, w.dtype), Kr[off[b]:off[b + 1]], w.dtype, "projected K")
                _assert_out_close(R.widen(Vg, w.dtype), Vr[off[b]:off[b + 1]], w.dtype, "projected V")

    if w.dtype == "bf16":
        # the same decisions applied to another cache (shared across layers) reproduce the pages bit for bit
        g4 = h.GpuPath(w, pre, pred)
        P.dllava_compact(w.B, g.seq_off, out["kept_idx"], out["out_off"], w.sumN, None, None, 0, None, None, g.pre["K"],
                         g.pre["V"], g4.cache, g4.err, g4.code)
        assert torch.equal(g4.pages, g.pages) and torch.equal(g4.cache_len, g.cache_len)
        # training form (Eq. 7) on the full token set with the selection's mask
        Om = torch.zeros_like(g.pre["Q"])
        wsm = torch.empty(P.dllava_masked_attn_workspace(w.sumN, w.B), dtype=torch.uint8, device=h.DEV)
        P.dllava_masked_attn(g.pre["Q"], g.pre["K"], g.pre["V"], w.B, g.seq_off, w.sumN, w.H, w.Dh, g.scale,
                             out["keep_mask"], Om, g.code, wsm)
        _assert_out_close(h.as_f64(Om), R.masked_attn(pre["Q"], pre["K"], pre["V"], w.seq_off, mask, g.scale, w.dtype),
                          w.dtype, "masked attention")
        # predictors in the appendix's form: image spans, and the rows of the first decode step
        from oracle import predictor_ref as PR
        from tests.test_gpu_predictor import image_tol, upload
        for nb in (2, 0):
            Pw = W.paper_predictor(w, nb)
            spans = nb == 2
            M = len(vis) if spans else w.B
            if M == 0:
                continue
            Dp = torch.zeros((M, 2), dtype=torch.float32, device=h.DEV)
            wsp = torch.empty(P.dllava_predict_workspace(M, w.B, nb), dtype=torch.uint8, device=h.DEV)
            if spans:
                P.dllava_predict(g.pre["hidden"], w.d, M, w.B, g.seq_off, g.vis_start, g.vis_len, upload(h, Pw, w.d), P.BF16,
                                 Dp, wsp)
                ref = PR.predict(pre["hidden"][vis], np.concatenate([[0], np.cumsum(w.n_vis)]), Pw, "bf16")
            else:
                P.dllava_predict(h.to_dev(dec["x"][0], "bf16"), w.d, M, 0, None, None, None, upload(h, Pw, w.d), P.BF16,
                                 Dp, wsp)
                ref = PR.predict(dec["x"][0], None, Pw, "bf16")
            tol = image_tol(pre["hidden"][vis], np.concatenate([[0], np.cumsum(w.n_vis)]), Pw, ref) if spans else TOL
            assert np.abs(Dp.cpu().numpy() - ref).max() <= tol

    # decode, both forms, with forced decisions (a seeded pattern): outputs close, caches bit-exact
    pattern = W.keep_pattern(w, w.T)
    g3 = h.GpuPath(w, pre, pred)
    g3.select_compact(torch.from_numpy(D_ref).to(h.DEV))
    ws = torch.zeros(P.dllava_decode_step_workspace(w.B, w.H, w.Dh, g3.cache.max_pages_per_seq, w.d, w.dh, g3.code),
                     dtype=torch.uint8, device=h.DEV)
    dev = {n: h.to_dev(dec[n], w.dtype) for n in ("x", "q", "k", "v")}
    logits = torch.zeros((w.T, w.B, 2), dtype=torch.float32, device=h.DEV)
    p = g3.pred
    for t in range(w.T):
        ov = torch.from_numpy(pattern[t]).to(h.DEV)
        o, keep = g.decode(dev["q"][t], dev["k"][t], dev["v"][t], keep_override=ov)
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], pattern[t], cache, g.scale)
        assert not err.any()
        _assert_out_close(h.as_f64(o), o_ref, w.dtype, f"decode {t}")
        assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
        prev = t > 0
        o2 = torch.zeros_like(o)
        P.dllava_decode_step(dev["x"][t], w.d, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], dev["q"][t], dev["k"][t],
                             dev["v"][t], dev["k"][t - 1] if prev else None, dev["v"][t - 1] if prev else None, None,
                             torch.from_numpy(pattern[t - 1]).to(h.DEV) if prev else None, w.B, 0.0, g3.cache, g3.scale,
                             o2, logits[t], None, g3.err, ws)
        _assert_out_close(h.as_f64(o2), o_ref, w.dtype, f"deferred decode {t}")
        Dr = R.score(dec["x"][t], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
        assert np.abs(logits[t].cpu().numpy() - Dr).max() <= tol
    P.dllava_decode_commit(dev["k"][w.T - 1], dev["v"][w.T - 1], None, torch.from_numpy(pattern[w.T - 1]).to(h.DEV), w.B,
                           0.0, g3.cache, None, g3.err)
    assert np.array_equal(h.bits(g.pages), cache.pages)
    assert np.array_equal(h.bits(g3.pages), cache.pages)
    assert np.array_equal(g3.cache_len.cpu().numpy(), cache.cache_len)
    assert int(g.err.item()) == 0 and int(g3.err.item()) == 0
