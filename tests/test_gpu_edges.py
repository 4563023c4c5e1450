"""GPU edge cases, determinism, buffer overruns and HIP-graph replay for the four entry points."""
import math

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


def test_degenerate_sequences_in_a_batch():
    """Empty sequence, sequence without vision tokens, vision-only sequence, single-token sequence, k = 0."""
    h = _H()
    w = W.make("degenerate", "bf16", 256, 2, 128, 6, [0, 5, 0, 1, 0, 3], [0, 0, 17, 0, 1, 2], [0, 4, 0, 0, 0, 6], 0.4, 5,
               project_qkv=True)
    pre, pred = W.prefill_inputs(w), W.predictor(w)
    g = h.GpuPath(w, pre, pred, extra_tokens=8)
    D = g.score_vision()
    rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                           for b in range(w.B)]).astype(np.int64)
    D_ref = R.score(pre["hidden"][rows], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    assert np.abs(D.cpu().numpy() - D_ref).max() <= TOL
    out = g.select_compact(torch.from_numpy(D_ref).to(h.DEV))
    mask, idx, off = R.select(D_ref, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    total = int(off[-1])
    assert list(np.diff(off)) == [0, 9, 6, 1, 0, 9]
    assert np.array_equal(out["out_off"].cpu().numpy(), off)
    assert np.array_equal(out["keep_mask"].cpu().numpy(), mask)
    assert np.array_equal(out["kept_idx"].cpu().numpy()[:total], idx)
    cache = R.PagedCache(g.pages.shape[0], g.bt_np, w.H, w.Dh, w.dtype)
    _, Qc = R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    assert np.array_equal(h.bits(g.pages), cache.pages)
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)]).astype(np.int64)
    O = g.prefill(out["Q_out"][:total].contiguous(), out["out_off"])
    O_ref = R.prefill_attn(Qc, pre["K"][src], pre["V"][src], off, g.scale, w.dtype)
    _assert_out_close(h.as_f64(O), O_ref, w.dtype, "prefill")
    # decode from ragged lengths that include two empty caches
    dec = W.decode_inputs(w)
    pattern = W.keep_pattern(w, w.T)
    for t in range(w.T):
        q, k, v = (h.to_dev(dec[n][t], w.dtype) for n in ("q", "k", "v"))
        o, keep = g.decode(q, k, v, keep_override=torch.from_numpy(pattern[t]).to(h.DEV))
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], pattern[t], cache, g.scale)
        assert not err.any()
        assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
        _assert_out_close(h.as_f64(o), o_ref, w.dtype, f"decode {t}")
    assert np.array_equal(h.bits(g.pages), cache.pages)


@pytest.mark.parametrize("B,H,Dh", [(1, 1, 64), (3, 5, 128), (64, 2, 64), (2, 40, 128)])
def test_decode_shapes_and_ragged_lengths(B, H, Dh):
    """Odd head counts, the largest batch the scoring fast path takes, several splits (small B*H) and none."""
    h = _H()
    T = 3
    w = W.make("shapes", "bf16", 256, H, Dh, B, 0, 0, 0, 1.0, T)
    rs = np.random.RandomState(B * 100 + H)
    lens = rs.randint(0, 150, size=B).astype(np.int32)
    lens[0] = 0
    mp = (int(lens.max()) + T) // 16 + 2
    bt = rng.permutation(7, "bt", B * mp).reshape(B, mp).astype(np.int32)
    g = h.GpuPath(w, None, None, n_pages=B * mp, bt=bt)
    pages_np = W.store(rng.normal(7, f"pages{B}{H}", (B * mp, 2, H, 16, Dh)), "bf16")
    g.pages.copy_(h.to_dev(pages_np, "bf16"))
    g.cache_len.copy_(torch.from_numpy(lens))
    cache = R.PagedCache(B * mp, bt, H, Dh, "bf16")
    cache.pages[...] = pages_np
    cache.cache_len[...] = lens
    dec = W.decode_inputs(w, T)
    for t in range(T):
        keep = rng.bernoulli(7, f"keep{t}", (B,), 0.5)
        q, k, v = (h.to_dev(dec[n][t], "bf16") for n in ("q", "k", "v"))
        o, ko = g.decode(q, k, v, keep_override=torch.from_numpy(keep).to(h.DEV))
        o_ref, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep, cache, g.scale)
        assert not err.any() and np.array_equal(ko.cpu().numpy(), keep)
        assert np.array_equal(g.cache_len.cpu().numpy(), cache.cache_len)
        _assert_out_close(h.as_f64(o), o_ref, "bf16", f"step {t}")
    assert np.array_equal(h.bits(g.pages), cache.pages)


@pytest.mark.parametrize("waves,splits", [(4, 1), (8, 1), (4, 3), (8, 2), (8, 16)])
def test_decode_launch_shapes_forced(waves, splits):
    """Every decode launch shape (waves per block, blocks per (sequence, head)) on the same ragged input, through both
    forms of the step: the outputs and the cache must not depend on the shape the library would have picked."""
    from tests.test_gpu_decode_step import _run
    P.dllava_set_launch_override(P.LAUNCH_DECODE_WAVES, waves)
    P.dllava_set_launch_override(P.LAUNCH_DECODE_SPLITS, splits)
    try:
        test_decode_shapes_and_ragged_lengths(3, 5, 128)
        w = W.make("forced", "bf16", 256, 3, 128, 5, [70, 1, 16, 0, 33], 0, 0, 1.0, 6, project_qkv=True)
        _run(w, 6, 0.0, use_override=True)
        if splits <= 2:   # long caches: every wave walks several pages with ragged ends, both head sizes
            for Dh in (128, 64):
                w = W.make("forcedlong", "bf16", 256, 2, Dh, 4, [700, 333, 64, 129], 0, 0, 1.0, 4, project_qkv=True)
                _run(w, 4, 0.0, use_override=True)
    finally:
        P.dllava_set_launch_override(P.LAUNCH_DECODE_WAVES, 0)
        P.dllava_set_launch_override(P.LAUNCH_DECODE_SPLITS, 0)


@pytest.mark.parametrize("M", [1, 15, 16, 17, 33, 64, 65, 129])
def test_score_row_counts_around_the_kernel_switches(M):
    h = _H()
    w = W.make("rows", "bf16", 512, 4, 128, 1, 0, M, 0, 1.0, 0)
    pre, pred = W.prefill_inputs(w), W.predictor(w, random_bias=True)
    g = h.GpuPath(w, pre, pred)
    ref = R.score(pre["hidden"], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    assert np.abs(g.score_rows(g.pre["hidden"]).cpu().numpy() - ref).max() <= TOL
    assert np.abs(g.score_vision().cpu().numpy() - ref).max() <= TOL


@pytest.mark.parametrize("tile", [1, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("d,dh", [(512, 320), (64, 40), (4096, 1024)])
def test_score_tiles_forced(tile, d, dh):
    """Every tile shape of the many-rows scoring kernels on the same ragged spans (the library picks by problem size;
    dllava_set_launch_override forces each): token counts that end inside a tile, unit counts that end inside a unit
    tile (320 = 256 + 64, 40), one and many stages of d, random biases."""
    h = _H()
    w = W.make("tiles", "bf16", d, max(1, d // 128), 128 if d >= 128 else 64, 3, [3, 0, 5], [300, 77, 200], [2, 1, 0], 1.0, 0)
    w.dh = dh
    pre, pred = W.prefill_inputs(w), W.predictor(w, random_bias=True)
    g = h.GpuPath(w, pre, pred)
    rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                           for b in range(w.B)])
    ref = R.score(pre["hidden"][rows], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    P.dllava_set_launch_override(P.LAUNCH_SCORE_TILE, tile)
    try:
        got = g.score_vision().cpu().numpy()
        again = g.score_vision().cpu().numpy()
        plain = g.score_rows(g.pre["hidden"]).cpu().numpy()
    finally:
        P.dllava_set_launch_override(P.LAUNCH_SCORE_TILE, 0)
    assert np.abs(got - ref).max() <= TOL, np.abs(got - ref).max()
    assert np.array_equal(got, again)
    ref_all = R.score(pre["hidden"], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    assert np.abs(plain - ref_all).max() <= TOL


@pytest.mark.parametrize("B", [300, 1024, 1100])
@pytest.mark.parametrize("tile", [1, 4])
def test_score_many_short_spans(B, tile):
    """The block-level row mapping (span table in LDS): hundreds of sequences with spans of 0..9 vision tokens, so
    one token tile gathers rows from dozens of spans, some empty; 1024 sequences fill the table exactly and 1100
    exceed it (the per-row search serves those).  Both many-rows kernels."""
    h = _H()
    rs = np.random.RandomState(B)
    n_vis = [int(v) for v in rs.randint(0, 10, size=B)]
    n_vis[0] = 0
    n_vis[-1] = 0
    n_sys = [int(v) for v in rs.randint(0, 3, size=B)]
    n_txt = [int(v) for v in rs.randint(0, 3, size=B)]
    w = W.make("spans", "bf16", 128, 1, 128, B, n_sys, n_vis, n_txt, 1.0, 0)
    w.dh = 320
    pre, pred = W.prefill_inputs(w), W.predictor(w, random_bias=True)
    g = h.GpuPath(w, pre, pred)
    rows = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                           for b in range(w.B)])
    assert len(rows) > 1000
    ref = R.score(pre["hidden"][rows], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    P.dllava_set_launch_override(P.LAUNCH_SCORE_TILE, tile)
    try:
        got = g.score_vision().cpu().numpy()
    finally:
        P.dllava_set_launch_override(P.LAUNCH_SCORE_TILE, 0)
    assert np.abs(got - ref).max() <= TOL, np.abs(got - ref).max()


@pytest.mark.parametrize("first", ["prefill", "decode"])
def test_score_forms_share_one_workspace(first):
    """A workspace sized for the largest row count serves every smaller one: the tiled form (576 vision rows) and the
    few-rows form (16 and 40 rows) alternate on ONE zero-filled buffer at the 7B predictor shape, in both orders."""
    h = _H()
    w = W.make("sharews", "bf16", 4096, 1, 128, 1, 0, 576, 0, 1.0, 0)
    pre, pred = W.prefill_inputs(w), W.predictor(w, random_bias=True)
    g = h.GpuPath(w, pre, pred)
    ref = R.score(pre["hidden"], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    ws = torch.zeros(P.dllava_score_workspace(576, w.d, w.dh, g.code), dtype=torch.uint8, device=h.DEV)
    p = g.pred

    def run(M):
        out = torch.full((M, 2), float("nan"), dtype=torch.float32, device=h.DEV)
        P.dllava_score(g.pre["hidden"], w.d, M, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"],
                       g.code, out, ws)
        assert np.abs(out.cpu().numpy() - ref[:M]).max() <= TOL, M

    order = [576, 16, 576, 40, 16, 576] if first == "prefill" else [16, 576, 40, 576, 16]
    for M in order:
        run(M)


@pytest.mark.parametrize("d", [64, 192, 320])
def test_score_odd_number_of_pipeline_stages(d):
    """The tiled scoring kernel pairs its 64-element stages; d = 64, 192, 320 leave an unpaired last stage."""
    h = _H()
    w = W.make("stages", "bf16", d, d // 64, 64, 1, 3, 200, 2, 1.0, 0)
    pre, pred = W.prefill_inputs(w), W.predictor(w, random_bias=True)
    g = h.GpuPath(w, pre, pred)
    ref = R.score(pre["hidden"], pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    assert np.abs(g.score_rows(g.pre["hidden"]).cpu().numpy() - ref).max() <= TOL
    vis = slice(3, 203)
    assert np.abs(g.score_vision().cpu().numpy() - ref[vis]).max() <= TOL


@pytest.mark.parametrize("waves", [1, 2, 4])
@pytest.mark.parametrize("from_cache", [False, True])
def test_prefill_tile_widths(waves, from_cache):
    """The matrix-core prefill kernel with 32, 64 and 128 queries per block (the library picks by problem size;
    dllava_set_launch_override forces each), ragged sequence lengths around the tile sizes."""
    h = _H()
    import paper_2412_00876_amd as P
    P.dllava_set_launch_override(P.LAUNCH_PREFILL_WAVES, waves)
    try:
        _prefill_tile_widths(h, waves, from_cache)
    finally:
        P.dllava_set_launch_override(P.LAUNCH_PREFILL_WAVES, 0)


def _prefill_tile_widths(h, waves, from_cache):
    B = 6
    w = W.make("widths", "bf16", 512, 4, 128, B, 0, [1, 31, 33, 64, 129, 200], 0, 1.0, 0)
    pre = W.prefill_inputs(w)
    g = h.GpuPath(w, pre, None)
    D = rng.normal(w.seed, "w.D", (int(sum(w.n_vis)), 2)).astype(np.float32)
    out = g.select_compact(torch.from_numpy(D).to(h.DEV), with_hidden=False)
    off = np.asarray(w.seq_off, np.int32)
    ref = R.prefill_attn(pre["Q"], pre["K"], pre["V"], off, g.scale, w.dtype)
    Qc = out["Q_out"].contiguous()
    if from_cache:
        O = g.prefill(Qc, out["out_off"])
    else:
        O = g.prefill(Qc, out["out_off"], g.pre["K"], g.pre["V"])
    _assert_out_close(h.as_f64(O), ref, w.dtype, f"prefill {waves} waves")


@pytest.mark.parametrize("B,Dh,lens", [
    (7, 128, [300, 1, 129, 0, 257, 40, 128]),      # ragged, an empty sequence in the middle: block numbering by tile index
    (70, 128, None),                                # more sequences than lanes of a wave: numbering sequence by sequence
    (5, 64, [130, 33, 0, 64, 97]),                  # the smaller head size
])
@pytest.mark.parametrize("from_cache", [False, True])
def test_prefill_block_numbering(B, Dh, lens, from_cache):
    """Blocks of the matrix-core prefill kernel are numbered by descending query-tile index over all sequences
    (each wave works out which (sequence, tile) it serves): every row of every sequence must still be produced
    exactly once, whatever the mix of lengths."""
    h = _H()
    if lens is None:
        lens = [1 + (37 * i) % 90 for i in range(B)]
    w = W.make("numbering", "bf16", 256, 2, Dh, B, 0, lens, 0, 1.0, 0)
    pre = W.prefill_inputs(w)
    g = h.GpuPath(w, pre, None)
    D = rng.normal(w.seed, "w.D", (int(sum(w.n_vis)), 2)).astype(np.float32)
    out = g.select_compact(torch.from_numpy(D).to(h.DEV), with_hidden=False)
    off = np.asarray(w.seq_off, np.int32)
    ref = R.prefill_attn(pre["Q"], pre["K"], pre["V"], off, g.scale, w.dtype)
    Qc = out["Q_out"].contiguous()
    if from_cache:
        O = g.prefill(Qc, out["out_off"])
    else:
        O = g.prefill(Qc, out["out_off"], g.pre["K"], g.pre["V"])
    _assert_out_close(h.as_f64(O), ref, w.dtype, f"prefill numbering B={B} Dh={Dh}")


@pytest.mark.parametrize("blocks", [1, 3, 7])
@pytest.mark.parametrize("waves", [1, 2, 4])
@pytest.mark.parametrize("from_cache", [False, True])
def test_prefill_persistent_blocks_walk_many_items(blocks, waves, from_cache):
    """The blocks of the matrix-core prefill kernel are persistent: each takes every `blocks`-th work item and streams
    their key tiles across the item boundaries (tile loads two tiles ahead, the next item's queries requested during
    the current item's last tile, outputs stored one tile late).  With 1, 3 or 7 blocks forced, every block walks
    many items of all lengths: one-tile items, an empty sequence, sequences that end inside a tile."""
    h = _H()
    lens = [300, 1, 129, 0, 257, 40, 128, 33, 64, 5]
    P.dllava_set_launch_override(P.LAUNCH_PREFILL_BLOCKS, blocks)
    P.dllava_set_launch_override(P.LAUNCH_PREFILL_WAVES, waves)
    try:
        w = W.make("persistent", "bf16", 384, 3, 128, len(lens), 0, lens, 0, 1.0, 0)
        pre = W.prefill_inputs(w)
        g = h.GpuPath(w, pre, None)
        D = rng.normal(w.seed, "w.D", (int(sum(w.n_vis)), 2)).astype(np.float32)
        out = g.select_compact(torch.from_numpy(D).to(h.DEV), with_hidden=False)
        off = np.asarray(w.seq_off, np.int32)
        ref = R.prefill_attn(pre["Q"], pre["K"], pre["V"], off, g.scale, w.dtype)
        Qc = out["Q_out"].contiguous()
        O = g.prefill(Qc, out["out_off"]) if from_cache else g.prefill(Qc, out["out_off"], g.pre["K"], g.pre["V"])
        again = g.prefill(Qc, out["out_off"]) if from_cache else g.prefill(Qc, out["out_off"], g.pre["K"], g.pre["V"])
    finally:
        P.dllava_set_launch_override(P.LAUNCH_PREFILL_BLOCKS, 0)
        P.dllava_set_launch_override(P.LAUNCH_PREFILL_WAVES, 0)
    _assert_out_close(h.as_f64(O), ref, w.dtype, f"prefill {blocks} blocks, {waves} waves")
    assert torch.equal(O.view(torch.int16), again.view(torch.int16))


def test_prefill_long_sequences_from_pages():
    """Sequences of more than 1024 keys (more than 64 pages each) read from the paged cache: the result must equal, bit
    for bit, the one computed from plain K/V rows, and match the oracle (the context a decoding step without KV cache
    reaches: reduced prompt plus a thousand generated tokens)."""
    h = _H()
    lens = [1238, 1030, 70]
    w = W.make("longpaged", "bf16", 256, 2, 128, len(lens), 0, lens, 0, 1.0, 0)
    pre = W.prefill_inputs(w)
    g = h.GpuPath(w, pre, None)
    D = rng.normal(w.seed, "w.D", (int(sum(w.n_vis)), 2)).astype(np.float32)
    out = g.select_compact(torch.from_numpy(D).to(h.DEV), with_hidden=False)
    off = np.asarray(w.seq_off, np.int32)
    Qc = out["Q_out"].contiguous()
    O_pages = g.prefill(Qc, out["out_off"])
    O_rows = g.prefill(Qc, out["out_off"], g.pre["K"], g.pre["V"])
    assert torch.equal(O_pages.view(torch.int16), O_rows.view(torch.int16))
    ref = R.prefill_attn(pre["Q"], pre["K"], pre["V"], off, g.scale, w.dtype)
    _assert_out_close(h.as_f64(O_pages), ref, w.dtype, "long sequences from pages")


@pytest.mark.parametrize("theta", [0.0, 0.4, float("inf"), float("-inf")])
def test_decode_step_without_kv_cache(theta):
    """Decoding without KV cache (Sec. 3.3.2, Eq. 12): every sequence is its reduced prompt followed by all output
    tokens so far; the output span is masked by the threshold rule with its last token always kept, compacted, and
    attended causally.  Mask, indices and offsets bit-exact, attention rows within the output tolerance."""
    h = _H()
    import paper_2412_00876_amd as P
    n_p, n_ot = [37, 0, 130, 5, 64], [9, 3, 1, 0, 150]      # a sequence without prompt, one without output tokens
    w = W.make("nocache", "bf16", 256, 3, 128, 5, n_p, n_ot, 0, 1.0, 0)
    pre = W.prefill_inputs(w)
    g = h.GpuPath(w, pre, None)
    D = rng.normal(w.seed, "ot.D", (int(sum(n_ot)), 2)).astype(np.float32)
    out = g.select_compact(torch.from_numpy(D).to(h.DEV), mode=P.MODE_THRESHOLD_KEEP_LAST, theta=theta, with_hidden=False)
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.THRESHOLD_KEEP_LAST, 0.0, theta)
    total = int(off[-1])
    assert np.array_equal(out["keep_mask"].cpu().numpy(), mask)
    assert np.array_equal(out["out_off"].cpu().numpy(), off)
    assert np.array_equal(out["kept_idx"].cpu().numpy()[:total], idx)
    for b in range(w.B):                       # the last output token of every sequence that has one is kept
        if n_ot[b]:
            assert mask[w.seq_off[b + 1] - 1] == 1
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)])
    O_ref = R.prefill_attn(pre["Q"][src], pre["K"][src], pre["V"][src], off, g.scale, w.dtype)
    O = g.prefill(out["Q_out"].contiguous(), out["out_off"])
    _assert_out_close(h.as_f64(O[:total]), O_ref, w.dtype, "attention over the reduced prompt and output tokens")


def test_results_are_bit_reproducible():
    """Every reduction runs in a fixed order (or in integer arithmetic): repeating a call must not change a bit."""
    h = _H()
    w = W.config(1)
    w.T = 6
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w)
    runs = []
    for _ in range(3):
        g = h.GpuPath(w, pre, pred)
        D = g.score_vision()
        out = g.select_compact(D)
        total = int(out["out_off"][-1].item())
        O = g.prefill(out["Q_out"][:total].contiguous(), out["out_off"])
        outs = [D.clone(), O.view(torch.int16).clone()]
        for t in range(w.T):
            x = h.to_dev(dec["x"][t], w.dtype)
            q, k, v = (h.to_dev(dec[n][t], w.dtype) for n in ("q", "k", "v"))
            Dt = g.score_rows(x)
            o, keep = g.decode(q, k, v, logits=Dt, theta=0.0)
            outs += [Dt.clone(), o.view(torch.int16).clone(), keep.clone()]
        outs.append(g.pages.view(torch.int16).clone())
        runs.append(outs)
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(a, b)


def test_outputs_stay_inside_their_buffers():
    """Guard regions around every output keep their sentinel."""
    h = _H()
    w = W.make("guard", "bf16", 256, 3, 128, 2, [2, 1], [30, 21], [5, 0], 0.5, 2, project_qkv=True)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w)
    g = h.GpuPath(w, pre, pred)
    G = 64

    def guarded(n, dtype, fill):
        buf = torch.full((n + 2 * G,), fill, dtype=dtype, device=h.DEV)
        return buf, buf[G:G + n]

    M = int(sum(w.n_vis))
    lbuf, logits = guarded(2 * M, torch.float32, 777.0)
    p = g.pred
    P.dllava_score(g.pre["hidden"], w.d, M, w.B, g.seq_off, g.vis_start, g.vis_len, w.d, w.dh, p["W1"], p["b1"], p["W2"],
                   p["b2"], g.code, logits, g.ws_score)
    kept = int(sum(w.kept_len))
    mbuf, mask = guarded(w.sumN, torch.uint8, 99)
    ibuf, kidx = guarded(w.sumN, torch.int32, -5)
    obuf, off = guarded(w.B + 1, torch.int32, -5)
    hbuf, hout = guarded(kept * w.d, torch.bfloat16, 3.0)
    qbuf, qout = guarded(kept * w.H * w.Dh, torch.bfloat16, 3.0)
    P.dllava_select_compact(logits, w.B, g.seq_off, g.vis_start, g.vis_len, w.sumN, P.MODE_TOPK, w.keep_ratio, 0.0,
                            g.pre["hidden"], hout, w.d, g.pre["Q"], qout, g.pre["K"], g.pre["V"], g.cache, mask, kidx, off,
                            g.err, g.code, g.ws_select)
    Obuf, O = guarded(kept * w.H * w.Dh, torch.bfloat16, 3.0)
    P.dllava_prefill_attn(qout, None, None, g.cache, w.B, off, kept, w.H, w.Dh, g.scale, O, g.code)
    dbuf, o = guarded(w.B * w.H * w.Dh, torch.bfloat16, 3.0)
    kbuf, keep = guarded(w.B, torch.uint8, 99)
    q, k, v = (h.to_dev(dec[n][0], w.dtype) for n in ("q", "k", "v"))
    ov = torch.ones(w.B, dtype=torch.uint8, device=h.DEV)
    P.dllava_decode_attn_append(q, k, v, w.B, None, 0.0, ov, g.cache, g.scale, o, keep, g.err, g.ws_decode)
    torch.cuda.synchronize()
    for buf, fill in ((lbuf, 777.0), (mbuf, 99), (ibuf, -5), (obuf, -5), (hbuf, 3.0), (qbuf, 3.0), (Obuf, 3.0), (dbuf, 3.0),
                      (kbuf, 99)):
        assert bool((buf[:G] == fill).all()) and bool((buf[-G:] == fill).all())
    assert int(kidx[kept - 1].item()) >= 0 and bool((kidx[kept:] == -5).all())     # only sum N* entries are written


def test_decode_loop_replays_from_a_hip_graph():
    """The path never synchronises with the host, so a decode loop can be captured once and replayed.  Every replay,
    with eager work and synchronisations in between, must reproduce the eager result bit for bit."""
    h = _H()
    w = W.make("graph", "bf16", 512, 4, 128, 3, [2, 0, 1], [40, 25, 31], [6, 3, 9], 0.4, 12, project_qkv=True)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w)
    g = h.GpuPath(w, pre, pred)
    D = g.score_vision()
    x = h.to_dev(dec["x"], w.dtype)
    q, k, v = (h.to_dev(dec[n], w.dtype) for n in ("q", "k", "v"))
    T = w.T
    td = torch.bfloat16
    o = torch.zeros((T, w.B, w.H, w.Dh), dtype=td, device=h.DEV)
    lg = torch.zeros((T, w.B, 2), dtype=torch.float32, device=h.DEV)
    kp = torch.zeros((T, w.B), dtype=torch.uint8, device=h.DEV)
    mask = torch.zeros(w.sumN, dtype=torch.uint8, device=h.DEV)
    kidx = torch.zeros(w.sumN, dtype=torch.int32, device=h.DEV)
    off = torch.zeros(w.B + 1, dtype=torch.int32, device=h.DEV)
    p = g.pred

    def loop():
        P.dllava_select_compact(D, w.B, g.seq_off, g.vis_start, g.vis_len, w.sumN, P.MODE_TOPK, w.keep_ratio, 0.0, None, None,
                                w.d, None, None, g.pre["K"], g.pre["V"], g.cache, mask, kidx, off, g.err, g.code, g.ws_select)
        for t in range(T):
            P.dllava_score(x[t], w.d, w.B, 0, None, None, None, w.d, w.dh, p["W1"], p["b1"], p["W2"], p["b2"], g.code, lg[t],
                           g.ws_score_small)
            P.dllava_decode_attn_append(q[t], k[t], v[t], w.B, lg[t], 0.0, None, g.cache, g.scale, o[t], kp[t], g.err,
                                        g.ws_decode)

    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        loop()
        st.synchronize()
        ref = [o.view(torch.int16).clone(), lg.clone(), kp.clone(), g.pages.view(torch.int16).clone(), g.cache_len.clone()]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            loop()
        for rep in range(4):
            o.zero_(); lg.zero_(); kp.zero_()                # eager work between replays
            g.cache_len.fill_(12345)
            st.synchronize()
            graph.replay()
            st.synchronize()
            got = [o.view(torch.int16), lg, kp, g.pages.view(torch.int16), g.cache_len]
            for a, b in zip(ref, got):
                assert torch.equal(a, b), rep
    assert int(g.err.item()) == 0


def test_widened_entry_points_replay_from_a_hip_graph():
    """dllava_predict (both forms), dllava_masked_attn, dllava_compact, dllava_qkv_project and the no-scoring decode step
    captured once and replayed: every replay, with eager work and synchronisations in between, reproduces the eager
    result bit for bit (none of them synchronises with the host or relies on initialised workspace)."""
    from tests.test_gpu_predictor import upload
    h = _H()
    w = W.make("graph2", "bf16", 128, 4, 64, 3, [2, 0, 1], [70, 25, 40], [6, 3, 9], 0.4, 3, project_qkv=True, seed=99)
    pre, dec, pred = W.prefill_inputs(w), W.decode_inputs(w), W.predictor(w)
    g, g2 = h.GpuPath(w, pre, pred), h.GpuPath(w, pre, pred)
    M = int(sum(w.n_vis))
    img, txt = upload(h, W.paper_predictor(w, 2), w.d), upload(h, W.paper_predictor(w, 0), w.d)
    z8 = lambda n: torch.full((n,), 0x33, dtype=torch.uint8, device=h.DEV)
    ws_img, ws_txt = z8(P.dllava_predict_workspace(M, w.B, 2)), z8(P.dllava_predict_workspace(w.B, w.B, 0))
    ws_m = z8(P.dllava_masked_attn_workspace(w.sumN, w.B))
    ws_d = torch.zeros(P.dllava_decode_workspace(w.B, w.H, w.Dh, g.cache.max_pages_per_seq), dtype=torch.uint8, device=h.DEV)
    D = torch.zeros((M, 2), dtype=torch.float32, device=h.DEV)
    Dt = torch.zeros((w.T, w.B, 2), dtype=torch.float32, device=h.DEV)
    mask = torch.zeros(w.sumN, dtype=torch.uint8, device=h.DEV)
    kidx = torch.zeros(w.sumN, dtype=torch.int32, device=h.DEV)
    off = torch.zeros(w.B + 1, dtype=torch.int32, device=h.DEV)
    hid = torch.zeros((w.sumN, w.d), dtype=torch.bfloat16, device=h.DEV)
    Qp = torch.zeros((w.sumN, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
    Om = torch.zeros_like(g.pre["Q"])
    o = torch.zeros((w.T, w.B, w.H, w.Dh), dtype=torch.bfloat16, device=h.DEV)
    aw = {k: h.to_dev(v, "bf16") for k, v in W.attn_weights(w).items()}
    x, q, k, v = (h.to_dev(dec[n], "bf16") for n in ("x", "q", "k", "v"))

    def loop():
        P.dllava_predict(g.pre["hidden"], w.d, M, w.B, g.seq_off, g.vis_start, g.vis_len, img, P.BF16, D, ws_img)
        P.dllava_select_compact(D, w.B, g.seq_off, g.vis_start, g.vis_len, w.sumN, P.MODE_TOPK, w.keep_ratio, 0.0,
                                g.pre["hidden"], hid, w.d, None, None, None, None, None, mask, kidx, off, g.err, g.code,
                                g.ws_select)
        P.dllava_masked_attn(g.pre["Q"], g.pre["K"], g.pre["V"], w.B, g.seq_off, w.sumN, w.H, w.Dh, g.scale, mask, Om, P.BF16, ws_m)
        P.dllava_compact(w.B, g.seq_off, kidx, off, w.sumN, None, None, 0, None, None, g.pre["K"], g.pre["V"], g.cache, g.err,
                         g.code)
        P.dllava_qkv_project(hid, w.d, w.sumN, w.d, w.B, off, kidx, aw["q"], aw["k"], aw["v"], 10000.0, Qp, g2.cache, g2.err,
                             g2.code)
        for t in range(w.T):
            P.dllava_predict(x[t], w.d, w.B, 0, None, None, None, txt, P.BF16, Dt[t], ws_txt)
            P.dllava_decode_step(None, 0, 0, 0, None, None, None, None, q[t], k[t], v[t], k[t - 1] if t else None,
                                 v[t - 1] if t else None, Dt[t - 1] if t else None, None, w.B, 0.0, g.cache, g.scale, o[t],
                                 None, None, g.err, ws_d)

    outs = lambda: [D, Dt, mask, kidx, off, hid.view(torch.int16), Qp.view(torch.int16), Om.view(torch.int16),
                    o.view(torch.int16), g.pages.view(torch.int16), g.cache_len, g2.pages.view(torch.int16), g2.cache_len]
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        loop()
        st.synchronize()
        ref = [t.clone() for t in outs()]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            loop()
        for rep in range(3):
            for t in (D, Dt, Om, o, Qp, hid):
                t.zero_()                                      # eager work between replays
            g.cache_len.fill_(777); g2.cache_len.fill_(777)
            ws_img.fill_(rep); ws_txt.fill_(rep + 7); ws_m.fill_(rep + 9)
            st.synchronize()
            graph.replay()
            st.synchronize()
            for i, (a, b) in enumerate(zip(ref, outs())):
                assert torch.equal(a, b), (rep, i)
    assert int(g.err.item()) == 0 and int(g2.err.item()) == 0
