"""GPU parity of dllava_qkv_project (projection of the reduced set with rotary rotation, K/V into the pages)
against the oracle: small ragged batches through both kernels, the chain select -> project -> prefill attention,
capacity overflow, large positions, and the benchmark's full shape on sampled rows."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_parity import TOL, TOL_F32, _assert_out_close

ROPE = 10000.0


def _H():
    from tests import harness
    return harness


def _select_oracle(w, pre, pred):
    vis = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                          for b in range(w.B)]).astype(np.int64)
    D = R.score(pre["hidden"][vis], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    return D, idx, off


def _project_gpu(h, g, w, x_dev, off_dev, pos_dev, aw, rope_base, rows):
    Wd = {k: h.to_dev(v, w.dtype) for k, v in aw.items()}
    Q = torch.zeros((rows, w.H, w.Dh), dtype=h.tdtype(w.dtype), device=h.DEV)
    P.dllava_qkv_project(x_dev, x_dev.stride(0), rows, w.d, w.B, off_dev, pos_dev, Wd["q"], Wd["k"], Wd["v"],
                         rope_base, Q, g.cache, g.err, g.code)
    return Q


@pytest.mark.parametrize("dtype,d,H,Dh,rope_base", [
    ("bf16", 256, 3, 128, ROPE),    # matrix-core kernel, four stages of the hidden dimension
    ("bf16", 192, 2, 128, ROPE),    # odd number of stages
    ("bf16", 256, 3, 128, 0.0),     # no rotation
    ("bf16", 128, 4, 64, ROPE),     # generic kernel: the smaller head size
    ("f32", 128, 2, 64, ROPE),      # generic kernel: float32 storage
])
def test_projection_of_a_ragged_batch(dtype, d, H, Dh, rope_base):
    """select -> compact (hidden states only) -> project: Q rows, K/V in the pages and the cache lengths against
    the oracle, on sequences whose kept lengths straddle the 128-row tiles (and one empty sequence)."""
    _ragged_batch(dtype, d, H, Dh, rope_base)


def _ragged_batch(dtype, d, H, Dh, rope_base, chain=True):
    h = _H()
    w = W.make("qkv", dtype, d, H, Dh, 5, [3, 0, 0, 1, 2], [300, 17, 0, 260, 40], [30, 2, 0, 0, 9], 0.5, 0,
               project_qkv=True)
    pre, pred, aw = W.prefill_inputs(w), W.predictor(w), W.attn_weights(w)
    D, idx, off = _select_oracle(w, pre, pred)
    total = int(off[-1])
    g = h.GpuPath(w, pre, pred)
    out = g.select_compact(torch.from_numpy(D).to(h.DEV), with_q=False, with_kv=False)
    assert np.array_equal(out["out_off"].cpu().numpy(), off)
    assert (g.cache_len.cpu().numpy() == 0).all()   # compaction of hidden states only leaves the cache alone
    Q = _project_gpu(h, g, w, out["hidden_out"], out["out_off"], out["kept_idx"], aw, rope_base, w.sumN)

    h_star, _ = R.compact(idx, off, w.seq_off, hidden=pre["hidden"])
    bt, n_pages = W.block_table(w)
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    Qr, Kr, Vr = R.qkv_project(h_star, off, idx[:total], aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype,
                               rope_base if rope_base > 0 else None, cache)
    _assert_out_close(h.as_f64(Q[:total]), Qr, w.dtype, "Q")
    assert (h.as_f64(Q[total:]) == 0).all()
    assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
    assert int(g.err.item()) == 0
    for b in range(w.B):
        n = int(off[b + 1] - off[b])
        if n == 0:
            continue
        Kg, Vg = g.cache_rows(b, n)
        _assert_out_close(R.widen(Kg, w.dtype), Kr[off[b]:off[b + 1]], w.dtype, f"K of sequence {b}")
        _assert_out_close(R.widen(Vg, w.dtype), Vr[off[b]:off[b + 1]], w.dtype, f"V of sequence {b}")

    if not chain:
        return
    # the chain continues: attention over the projected, cached reduced set
    O = g.prefill(Q.contiguous(), out["out_off"])
    Ks, Vs = R.narrow(Kr, w.dtype), R.narrow(Vr, w.dtype)
    O_ref = R.prefill_attn(R.narrow(Qr, w.dtype), Ks, Vs, off, g.scale, w.dtype)
    err = np.abs(h.as_f64(O[:total]) - O_ref)
    # both sides round Q, K, V to the stored form on their own: a flat bar on the attention outputs
    assert err.max() <= (TOL if dtype == "bf16" else 10 * TOL_F32), float(err.max())


@pytest.mark.parametrize("tile", [1, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("H,d", [(3, 256), (4, 4096)])
def test_projection_tiles_forced(tile, H, d):
    """Every tile shape of the matrix-core projection kernels on the same ragged batch (the library picks by problem
    size; dllava_set_launch_override forces each): an odd head count (the last feature tile of the large-tile kernel
    holds one head only), kept lengths that end inside a token tile, few and many stages of d."""
    P.dllava_set_launch_override(P.LAUNCH_QKV_TILE, tile)
    try:
        # (the attention that follows is left to the small case: with d = 4096 its logits are sharp enough for the two
        # sides' separately rounded Q and K to move an output by more than the flat bar, whatever kernel projects)
        _ragged_batch("bf16", d, H, 128, ROPE, chain=d <= 256)
    finally:
        P.dllava_set_launch_override(P.LAUNCH_QKV_TILE, 0)


def test_projection_large_positions_and_strided_rows():
    """Positions up to 2^24 - 1 keep their full angle (the product position x frequency is reduced without
    losing its low bits); x may have a row stride larger than d."""
    h = _H()
    w = W.make("qkvpos", "bf16", 128, 2, 128, 2, 0, [6, 7], 0, 1.0, 0, project_qkv=True)
    pre, aw = W.prefill_inputs(w), W.attn_weights(w)
    g = h.GpuPath(w, pre, None)
    rows = w.sumN
    pos = np.array([0, 1, 4095, 4096, 65535, 1000003, 0, 2, 131071, 524288, 8388607, 16777215, 12345678], np.int32)
    off = np.asarray(w.seq_off, np.int32)
    xw = torch.zeros((rows, w.d + 64), dtype=torch.bfloat16, device=h.DEV)
    xw[:, :w.d] = g.pre["hidden"]
    x_view = xw[:, :w.d]
    Q = _project_gpu(h, g, w, x_view, torch.from_numpy(off).to(h.DEV), torch.from_numpy(pos).to(h.DEV), aw, ROPE, rows)
    Qr, Kr, Vr = R.qkv_project(pre["hidden"], off, pos, aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, ROPE)
    _assert_out_close(h.as_f64(Q), Qr, w.dtype, "Q at large positions")
    for b in range(w.B):
        Kg, Vg = g.cache_rows(b, int(off[b + 1] - off[b]))
        _assert_out_close(R.widen(Kg, w.dtype), Kr[off[b]:off[b + 1]], w.dtype, "K at large positions")
        _assert_out_close(R.widen(Vg, w.dtype), Vr[off[b]:off[b + 1]], w.dtype, "V")


@pytest.mark.parametrize("Dh", [128, 64])
def test_projection_beyond_cache_capacity(Dh):
    """A sequence longer than its page list: the flag is raised, the length is clamped, the rows that fit are
    written, nothing else in the pages is touched; Q is complete."""
    h = _H()
    w = W.make("qkvcap", "bf16", 128, 2, Dh, 2, 0, [40, 20], 0, 1.0, 0, project_qkv=True)
    pre, aw = W.prefill_inputs(w), W.attn_weights(w)
    mp = 2  # 32 slots per sequence
    bt = np.array([[3, 1], [0, 2]], np.int32)
    g = h.GpuPath(w, pre, None, n_pages=5, bt=bt)
    g.pages.fill_(7.0)
    off = np.asarray(w.seq_off, np.int32)
    pos = np.concatenate([np.arange(40), np.arange(20)]).astype(np.int32)
    Q = _project_gpu(h, g, w, g.pre["hidden"], torch.from_numpy(off).to(h.DEV), torch.from_numpy(pos).to(h.DEV), aw,
                     ROPE, w.sumN)
    Qr, Kr, Vr = R.qkv_project(pre["hidden"], off, pos, aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, ROPE)
    assert int(g.err.item()) == 1
    assert g.cache_len.cpu().numpy().tolist() == [32, 20]
    _assert_out_close(h.as_f64(Q), Qr, w.dtype, "Q")
    Kg, Vg = g.cache_rows(0, 32)
    _assert_out_close(R.widen(Kg, w.dtype), Kr[:32], w.dtype, "K rows that fit")
    Kg, Vg = g.cache_rows(1, 20)
    _assert_out_close(R.widen(Vg, w.dtype), Vr[40:60], w.dtype, "V of the second sequence")
    pg = h.as_f64(g.pages)
    assert (pg[4] == 7.0).all()                 # a page no sequence owns
    assert (pg[2][:, :, 4:, :] == 7.0).all()    # slots 20.. of the second sequence's second page


def test_projection_full_shape_sampled():
    """The any-resolution benchmark shape (8 x 704 kept rows, d = 4096, 32 heads): rows sampled from every
    region of the launch against the oracle; every cache row of one sequence against the GPU's own Q/K/V layout."""
    h = _H()
    w = W.config(4)
    rs = np.random.RandomState(7)
    aw = W.attn_weights(w)
    rows = sum(w.kept_len)
    off = np.concatenate([[0], np.cumsum(w.kept_len)]).astype(np.int32)
    x = W.store(rng.normal(w.seed, "qkv.x", (rows, w.d)).astype(np.float32), w.dtype)
    pos = np.concatenate([np.sort(rs.choice(3008, size=n, replace=False)) for n in w.kept_len]).astype(np.int32)
    g = h.GpuPath(w, None, None)
    Q = _project_gpu(h, g, w, h.to_dev(x, w.dtype), torch.from_numpy(off).to(h.DEV), torch.from_numpy(pos).to(h.DEV),
                     aw, ROPE, rows)
    assert np.array_equal(g.cache_len.cpu().numpy(), np.asarray(w.kept_len))
    pick = sorted(set([0, 127, 128, 703, 704, rows - 1] + [int(v) for v in rs.choice(rows, size=18, replace=False)]))
    sub_off = np.arange(len(pick) + 1, dtype=np.int32)
    Qr, Kr, Vr = R.qkv_project(x[pick], sub_off, pos[pick], aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, ROPE)
    _assert_out_close(h.as_f64(Q[pick]), Qr, w.dtype, "Q sampled")
    pg = g.pages
    for n, r in enumerate(pick):
        b = int(np.searchsorted(off, r, side="right") - 1)
        j = r - int(off[b])
        page, slot = int(g.bt_np[b, j // 16]), j % 16
        _assert_out_close(h.as_f64(pg[page, 0, :, slot, :]), Kr[n], w.dtype, f"K row {r}")
        _assert_out_close(h.as_f64(pg[page, 1, :, slot, :]), Vr[n], w.dtype, f"V row {r}")
