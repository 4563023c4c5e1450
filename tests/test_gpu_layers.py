"""The one-time decision shared by all later layers (Sec. 3.3; l = 2 in the paper): a stack of attention layers in which
layers 1..l keep full caches and layers l+1..L the reduced ones, driven through paper_2412_00876_amd.layers, against the
oracle applied layer by layer.  Also dllava_compact (compaction with decisions already taken) on its own."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_parity import _assert_out_close


def _H():
    from tests import harness
    return harness


def _layer_tensors(w, layer, T):
    seed = w.seed + 100 * (layer + 1)
    pre = {n: W.store(rng.normal(seed, n, (w.sumN, w.H, w.Dh)), w.dtype) for n in ("Q", "K", "V")}
    dec = {n: W.store(rng.normal(seed, "d" + n, (T, w.B, w.H, w.Dh)), w.dtype) for n in ("q", "k", "v")}
    return pre, dec


@pytest.mark.parametrize("L,l", [(4, 2), (3, 0), (2, 2)])
def test_layer_stack_shares_one_decision(L, l):
    from paper_2412_00876_amd.layers import SparsifiedLayers
    h = _H()
    T = 5
    w = W.make("stack", "bf16", 64, 2, 128, 3, [2, 0, 1], [40, 17, 70], [6, 3, 9], 0.3, T, seed=900 + L)
    pre0, pred = W.prefill_inputs(w), W.predictor(w)
    vis = np.concatenate([np.arange(w.seq_off[b] + w.vis_start[b], w.seq_off[b] + w.vis_start[b] + w.vis_len[b])
                          for b in range(w.B)]).astype(np.int64)
    D = R.score(pre0["hidden"][vis], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)   # after layer l
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    pattern = W.keep_pattern(w, T)                              # the shared decisions of the generated tokens
    scale = 1.0 / math.sqrt(w.Dh)
    n_full = np.diff(w.seq_off)
    full_idx = np.concatenate([np.arange(n) for n in n_full]).astype(np.int32)
    full_off = np.asarray(w.seq_off, np.int32)

    i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(h.DEV)
    cap_full = int(n_full.max()) + T
    cap_red = int(np.diff(off).max()) + T
    S = SparsifiedLayers(L, l, w.B, w.H, w.Dh, cap_full, cap_red, torch.bfloat16)
    S.begin(i32(w.seq_off), i32(w.vis_start), i32(w.vis_len), w.sumN)
    assert np.array_equal(S.full_idx.cpu().numpy(), full_idx) and np.array_equal(S.full_off.cpu().numpy(), full_off)
    Qs = torch.zeros((w.sumN, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
    kv_tokens = 0
    for layer in range(L):
        if layer == l:
            S.decide(torch.from_numpy(D).to(h.DEV), w.keep_ratio)
            assert np.array_equal(S.out_off.cpu().numpy(), off)
            assert np.array_equal(S.kept_idx.cpu().numpy()[:off[-1]], idx)
        pre, dec = _layer_tensors(w, layer, T)
        k_idx, k_off = (full_idx, full_off) if layer < l else (idx, off)
        total = int(k_off[-1])
        O = torch.zeros((w.sumN, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
        S.prefill_layer(layer, h.to_dev(pre["Q"], "bf16"), h.to_dev(pre["K"], "bf16"), h.to_dev(pre["V"], "bf16"), O, Qs)
        c = S.caches[layer]
        cache = R.PagedCache(c.pages.shape[0], c.block_table.cpu().numpy(), w.H, w.Dh, "bf16")
        _, Qc = R.compact(k_idx, k_off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
        assert np.array_equal(h.bits(c.pages), cache.pages), f"layer {layer}: pages after prefill"
        assert np.array_equal(c.cache_len.cpu().numpy(), cache.cache_len)
        src = np.concatenate([w.seq_off[b] + k_idx[k_off[b]:k_off[b + 1]] for b in range(w.B)])
        O_ref = R.prefill_attn(Qc, pre["K"][src], pre["V"][src], k_off, scale, "bf16")
        _assert_out_close(h.as_f64(O[:total]), O_ref, "bf16", f"layer {layer} prefill")
        for t in range(T):
            o = torch.zeros((w.B, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
            keep_t = np.ones(w.B, np.uint8) if layer < l else pattern[t]
            S.decode_layer(layer, h.to_dev(dec["q"][t], "bf16"), h.to_dev(dec["k"][t], "bf16"),
                           h.to_dev(dec["v"][t], "bf16"), o, torch.from_numpy(pattern[t]).to(h.DEV))
            o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep_t, cache, scale)
            assert not err.any()
            _assert_out_close(h.as_f64(o), o_ref, "bf16", f"layer {layer} step {t}")
        assert np.array_equal(h.bits(c.pages), cache.pages), f"layer {layer}: pages after decode"
        assert np.array_equal(c.cache_len.cpu().numpy(), cache.cache_len)
        kv_tokens += int(cache.cache_len.sum())
    assert int(S.err.item()) == 0
    # memory: l full layers (every prompt and generated token) + (L - l) reduced ones
    expect = l * int(n_full.sum() + T * w.B) + (L - l) * int(off[-1] + pattern.sum())
    assert kv_tokens == expect
    assert S.kv_bytes() == expect * 2 * w.H * w.Dh * 2


def test_compact_with_given_decisions_matches_select_compact():
    """dllava_compact with the kept_idx / out_off of an earlier dllava_select_compact call reproduces that call's
    outputs bit for bit (hidden, Q, pages, lengths), also when nothing is kept and beyond the capacity."""
    h = _H()
    w = W.make("cg", "bf16", 128, 2, 64, 3, [1, 0, 2], [30, 0, 50], [4, 0, 2], 0.4, 1, project_qkv=True, seed=77)
    pre, pred = W.prefill_inputs(w), W.predictor(w)
    g = h.GpuPath(w, pre, pred)
    D = g.score_vision()
    out = g.select_compact(D)
    g2 = h.GpuPath(w, pre, pred)
    hid2 = torch.zeros_like(out["hidden_out"])
    Q2 = torch.zeros_like(out["Q_out"])
    P.dllava_compact(w.B, g.seq_off, out["kept_idx"], out["out_off"], w.sumN, g.pre["hidden"], hid2, w.d, g.pre["Q"], Q2,
                     g.pre["K"], g.pre["V"], g2.cache, g2.err, g2.code)
    total = int(out["out_off"][-1].item())
    assert torch.equal(hid2[:total], out["hidden_out"][:total]) and torch.equal(Q2[:total], out["Q_out"][:total])
    assert torch.equal(g2.pages, g.pages) and torch.equal(g2.cache_len, g.cache_len)
    assert int(g2.err.item()) == 0
    # a cache too small for the kept rows: flagged, lengths clamped, nothing written past the capacity
    small_pages = torch.zeros((w.B * 1, 2, w.H, 16, w.Dh), dtype=torch.bfloat16, device=h.DEV)
    small = P.KVCache(small_pages, torch.arange(w.B, dtype=torch.int32, device=h.DEV).reshape(w.B, 1).contiguous(),
                      torch.zeros(w.B, dtype=torch.int32, device=h.DEV))
    err = torch.zeros(1, dtype=torch.int32, device=h.DEV)
    P.dllava_compact(w.B, g.seq_off, out["kept_idx"], out["out_off"], w.sumN, None, None, 0, None, None, g.pre["K"],
                     g.pre["V"], small, err, g.code)
    n_kept = np.diff(out["out_off"].cpu().numpy())
    assert int(err.item()) == 1 and np.array_equal(small.cache_len.cpu().numpy(), np.minimum(n_kept, 16))
