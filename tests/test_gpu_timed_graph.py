"""The very graph bench.py times (scoring, selection + compaction, prefill attention, every decode step as one launch
with the deferred append, the final commit), recorded once and replayed, against the oracle over the WHOLE run.

Integer work is compared in full at every step: the keep decision of every (step, sequence), the kept indices, the
final cache lengths and every byte of the pages after the last step.  Floating outputs are compared where the oracle
can follow: the decode logits of all sequences and the attention outputs of a few (sequence, head) pairs at the first
64 steps, the last 64 and every 16th (every 32nd of 2048) in between (the oracle's cache is advanced at EVERY step, so
a sampled step sees the cache exactly as long as the run made it).  Replays must agree with each other bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import dllava_ref as R
from synth import workloads as W
from tests.test_gpu_parity import TOL, _assert_out_close

FILL = 7.0   # pages start every replay from this value: a slot the run should have written cannot pass by being stale


def _H():
    from tests import harness
    return harness


def _pair_step(cache, b, hd, q, k_new, v_new, scale):
    """Oracle attention of one (sequence, head) at the cache's current length: the oracle's own decode step on that
    head's slice of the sequence's pages (heads and sequences do not interact in Eq. 6)."""
    L = int(cache.cache_len[b])
    used = (L + cache.page_size - 1) // cache.page_size
    one = R.PagedCache(max(used, 1), np.arange(max(used, 1), dtype=np.int32)[None], 1, cache.Dh, cache.dtype)
    if used:
        one.pages[:used] = cache.pages[cache.block_table[b, :used], :, hd:hd + 1]
    one.cache_len[0] = L
    o, _ = R.decode_attn_append(q[b:b + 1, hd:hd + 1], k_new[b:b + 1, hd:hd + 1], v_new[b:b + 1, hd:hd + 1],
                                np.zeros(1, np.uint8), one, scale)
    return o[0, 0]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("ci", [2, 3, 4])
def test_timed_graph_whole_run(ci):
    import bench
    h = _H()
    w = W.config(ci)
    path = bench.Path(w, torch, P, W)
    path.calibrate_theta()
    B, T, H = w.B, w.T, w.H
    pre, dec, pred = path.host["pre"], path.host["dec"], path.host["pred"]
    stream = torch.cuda.Stream()
    outs = ("logits_vis", "keep_mask", "kept_idx", "out_off", "hidden_out", "Q_out", "O", "logits_dec", "o_dec",
            "keep_dec", "pages", "cache_len")
    snaps = []
    with torch.cuda.stream(stream):
        path.step()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            path.step()
        for rep in range(2):
            for name in outs:                      # nothing a replay reports may be left over from the one before
                t = getattr(path, name)
                if name == "pages":
                    t.fill_(FILL)
                elif t.dtype.is_floating_point:
                    t.fill_(float("nan"))
                else:
                    t.fill_(113)
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            snaps.append({name: getattr(path, name).clone() for name in outs})
            # the program's own eager work between the replays: a different, shorter call sequence on the same buffers
            path.score_vision()
            path.select_compact()
            stream.synchronize()
    torch.cuda.synchronize()
    assert int(path.err.item()) == 0
    for name in outs:
        a, b = snaps[0][name], snaps[1][name]
        if a.dtype.is_floating_point:   # bit patterns, so NaN == NaN where a buffer is larger than what is written
            a, b = a.view(torch.int16 if a.element_size() == 2 else torch.int32), b.view(torch.int16 if b.element_size() == 2 else torch.int32)
        assert torch.equal(a, b), f"replays differ in {name}"
    s = snaps[1]
    rs = np.random.RandomState(900 + ci)

    # ---- prefill: logits on sampled rows, selection and compaction in full, from the GPU's logits
    D_np = s["logits_vis"].cpu().numpy()
    vis_rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                               for b in range(B)])
    pick = sorted(set([0, len(vis_rows) - 1] + [int(v) for v in rs.choice(len(vis_rows), 48, replace=False)]))
    ref = R.score(pre["hidden"][vis_rows[pick]], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    assert np.abs(D_np[pick] - ref).max() <= TOL
    mask, idx, off = R.select(D_np, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    total = int(off[-1])
    assert np.array_equal(s["out_off"].cpu().numpy(), off)
    assert np.array_equal(s["keep_mask"].cpu().numpy(), mask)
    assert np.array_equal(s["kept_idx"].cpu().numpy()[:total], idx)
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(B)])
    assert np.array_equal(h.bits(s["Q_out"])[:total], pre["Q"][src])
    cache = R.PagedCache(path.pages.shape[0], path.bt_np, H, w.Dh, w.dtype)
    cache.pages[...] = h.bits(torch.full((1,), FILL, dtype=path.pages.dtype))[0]
    R.compact(idx, off, w.seq_off, K=pre["K"], V=pre["V"], cache=cache)
    Oh = h.as_f64(s["O"])
    for _ in range(2):
        b, hd = int(rs.randint(B)), int(rs.randint(H))
        r0, r1 = int(off[b]), int(off[b + 1])
        Qc, Kc, Vc = pre["Q"][src[r0:r1], hd:hd + 1], pre["K"][src[r0:r1], hd:hd + 1], pre["V"][src[r0:r1], hd:hd + 1]
        o_ref = R.prefill_attn(Qc, Kc, Vc, np.array([0, r1 - r0]), path.scale, w.dtype)
        _assert_out_close(Oh[r0:r1, hd:hd + 1], o_ref, w.dtype, f"prefill b={b} h={hd}")

    # ---- decode: every step advances the oracle's cache; sampled steps are checked in floating point
    logits = s["logits_dec"].cpu().numpy()            # [T,B,2]
    keep_gpu = s["keep_dec"].cpu().numpy()            # [T,B]
    pairs = [(0, 0), (B - 1, H - 1)] + [(int(rs.randint(B)), int(rs.randint(H))) for _ in range(4)]
    stride = 16 if T <= 1024 else 32
    n_checked = n_firm = 0
    for t in range(T):
        keep_ref = R.decode_keep(logits[t], w.theta)                     # the decision rule, on the GPU's logits
        assert np.array_equal(keep_gpu[t], keep_ref), f"keep at step {t}"
        if t < 64 or t >= T - 64 or t % stride == 0:
            Dr = R.score(dec["x"][t], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
            assert np.abs(logits[t] - Dr).max() <= TOL, f"logits at step {t}"
            # ... and on the oracle's own logits wherever the margin is further from the threshold than the two
            # sides' logits may differ
            margin = Dr[:, 1] - Dr[:, 0]
            firm = np.abs(margin - w.theta) > 2 * TOL
            assert np.array_equal(keep_gpu[t][firm], R.decode_keep(Dr, w.theta)[firm]), f"firm keeps at step {t}"
            n_firm += int(firm.sum())
            o_t = h.as_f64(s["o_dec"][t])
            for b, hd in pairs:
                o_ref = _pair_step(cache, b, hd, dec["q"][t], dec["k"][t], dec["v"][t], path.scale)
                _assert_out_close(o_t[b, hd], o_ref, w.dtype, f"decode t={t} b={b} h={hd}")
            n_checked += 1
        _, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep_ref, cache, path.scale, only=[])
        assert not err.any()
    assert n_checked >= 128 and n_firm > n_checked * B // 2
    assert np.array_equal(s["cache_len"].cpu().numpy(), cache.cache_len)
    assert np.array_equal(cache.cache_len, np.asarray(w.kept_len) + keep_gpu.astype(np.int64).sum(0))
    assert np.array_equal(h.bits(s["pages"]), cache.pages)
