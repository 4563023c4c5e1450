"""GPU parity of the decoder-layer pieces beyond attention (dllava_rms_norm, the gated form of dllava_linear) to the
rounding of their outputs, and of a whole stack of LLaMA-family decoder layers with the one-time token reduction after
layer l (paper_2412_00876_amd.layers.DecoderStack) against the decoder-stack oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from oracle import decoder_ref as DR
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W
from tests.test_gpu_predictor import _assert_same_rounding


def _H():
    from tests import harness
    return harness


@pytest.mark.parametrize("M,d", [(50, 64), (33, 4096), (7, 5120), (9, 8192), (5, 520), (1500, 264), (1030, 8192)])
def test_rms_norm_layer(M, d):
    h = _H()
    x = W.store(rng.normal(d, "x", (M, d)) * 2 + 0.3, "bf16")
    g = rng.uniform(d, "g", (d,), 0.5, 1.5).astype(np.float32)
    y = torch.zeros((M, d + 8), dtype=torch.bfloat16, device=h.DEV)
    P.dllava_rms_norm(h.to_dev(x, "bf16"), d, M, d, torch.from_numpy(g).to(h.DEV), DR.RMS_EPS, y, d + 8, P.BF16)
    got = h.bits(y)
    assert (got[:, d:] == 0).all()
    _assert_same_rounding(got[:, :d], DR.rms_norm(R.widen(x, "bf16"), g), f"rms norm {M}x{d}")
    P.dllava_rms_norm(h.to_dev(x, "bf16"), d, M, d, None, DR.RMS_EPS, y, d + 8, P.BF16)
    _assert_same_rounding(h.bits(y)[:, :d], DR.rms_norm(R.widen(x, "bf16"), np.ones(d)), "rms norm without weight")


@pytest.mark.parametrize("M,K,N", [(130, 256, 704), (20, 64, 8)])
def test_gated_linear_layer(M, K, N):
    """y = (x W^T) * SiLU(gate): the second half of a SwiGLU feed-forward layer."""
    h = _H()
    x = W.store(rng.normal(K, "x", (M, K)), "bf16")
    Wm = W.store(rng.normal(K, "W", (N, K)) / np.sqrt(K), "bf16")
    gate = W.store(rng.normal(K, "g", (M, N)) * 2, "bf16")
    ref = (R.widen(x, "bf16") @ R.widen(Wm, "bf16").T) * DR.silu(R.widen(gate, "bf16"))
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=h.DEV)
    P.dllava_linear(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), None, N, 2, h.to_dev(gate, "bf16"), y, N, P.BF16)
    _assert_same_rounding(h.bits(y), ref, f"gated linear {M}x{K}x{N}")


def _upload_layers(h, layers):
    return [{k: (h.to_dev(v, "bf16") if v.dtype == np.uint16 else torch.from_numpy(v).to(h.DEV)) for k, v in L.items()}
            for L in layers]


@pytest.mark.parametrize("n_layers,l", [(3, 1), (2, 0), (2, 2)])
def test_decoder_stack_with_one_time_reduction(n_layers, l):
    from paper_2412_00876_amd.layers import DecoderStack
    h = _H()
    d, H, Dh, dff = 256, 2, 128, 512
    w = W.make("stack", "bf16", d, H, Dh, 3, [2, 0, 1], [40, 9, 70], [6, 3, 9], 0.3, 1, seed=500 + n_layers)
    layers = W.decoder_layers(w, n_layers, dff)
    pred = W.predictor(w)
    x0 = W.store(rng.normal(w.seed, "h0", (w.sumN, d)), "bf16")
    oracle_pred = lambda rows: R.score(rows, pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    xf, idx, off, logits_ref = DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, l, w.keep_ratio, oracle_pred,
                                                  H, Dh, "bf16")
    kept_rows = int(off[-1])
    M_vis = int(sum(w.n_vis))
    S = DecoderStack(_upload_layers(h, layers), l, w.B, H, Dh, d, dff, w.sumN, M_vis)
    i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(h.DEV)
    seq_off, vis_start, vis_len = i32(w.seq_off), i32(w.vis_start), i32(w.vis_len)
    pw = {k: (h.to_dev(v, "bf16") if v.dtype == np.uint16 else torch.from_numpy(v).to(h.DEV)) for k, v in pred.items()}
    ws = torch.zeros(P.dllava_score_workspace(M_vis, d, w.dh, P.BF16), dtype=torch.uint8, device=h.DEV)

    def predictor(X, logits):
        P.dllava_score(X, d, M_vis, w.B, seq_off, vis_start, vis_len, d, w.dh, pw["W1"], pw["b1"], pw["W2"], pw["b2"], P.BF16,
                       logits, ws)

    out = S.prefill(h.to_dev(x0, "bf16"), seq_off, vis_start, vis_len, w.keep_ratio, kept_rows if l < n_layers else w.sumN,
                    predictor)
    torch.cuda.synchronize()
    assert int(S.err.item()) == 0
    if l < n_layers:
        # the decision is taken on the GPU's own hidden states: its logits must agree with the oracle's closely enough
        # for the same tokens to be kept (checked, not assumed), and then the kept set is identical
        assert np.array_equal(S.out_off.cpu().numpy(), off)
        assert np.array_equal(S.kept_idx.cpu().numpy()[:kept_rows], idx[:kept_rows])
    got = h.as_f64(out)
    assert got.shape == xf.shape
    err = got - xf
    scale = np.sqrt(np.mean(xf ** 2))
    # a dozen bfloat16 tensors per layer: two correct evaluations settle about one rounding step apart (see the
    # predictor tests); a structural mistake (a missing residual, a wrong position) is of the order of the values
    assert np.sqrt(np.mean(err ** 2)) <= 2e-2 * scale, (np.sqrt(np.mean(err ** 2)), scale)
    assert np.abs(err).max() <= 0.15 * scale
    # K/V of the last layer's cache: the kept tokens only
    n_last = np.diff(off) if l < n_layers else np.diff(w.seq_off)
    assert np.array_equal(S.caches[-1].cache_len.cpu().numpy(), n_last)
    if l > 0:
        assert np.array_equal(S.caches[0].cache_len.cpu().numpy(), np.diff(w.seq_off))


@pytest.mark.parametrize("M,K,N,act,res", [(16, 4096, 4096, 0, "inplace"), (8, 4096, 11008, 2, "gate"), (40, 11008, 4096, 0, None),
                                            (1, 64, 32, 1, None), (64, 320, 96, 0, "other"), (20, 2048, 64, 1, "other"),
                                            (33, 4096, 128, 0, "inplace"), (32, 13824, 5120, 0, "other"),
                                            (32, 5120, 5120, 0, "inplace")])
def test_linear_layer_on_few_rows(M, K, N, act, res):
    h = _H()
    seed = 3000 + M + K + N
    x = W.store(rng.normal(seed, "x", (M, K)), "bf16")
    Wm = W.store(W._normal_big(seed, "W", (N, K)) / np.sqrt(K), "bf16")
    b = rng.uniform(seed, "b", (N,), -0.5, 0.5).astype(np.float32)
    r = W.store(rng.normal(seed, "r", (M, N)), "bf16") if res else None
    ref = R.widen(x, "bf16") @ R.widen(Wm, "bf16").T + b
    if act == 1:
        ref = R.gelu(ref)
    if res == "gate":
        ref = ref * DR.silu(R.widen(r, "bf16"))
    elif res:
        ref = ref + R.widen(r, "bf16")
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=h.DEV)
    rd = None
    if res == "inplace":
        y.copy_(h.to_dev(r, "bf16"))
        rd = y
    elif res:
        rd = h.to_dev(r, "bf16")
    ws = _few_workspace(P.dllava_linear_few_workspace(N, K), 0x44)
    P.dllava_linear_few(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), torch.from_numpy(b).to(h.DEV), N, act, rd, y, N,
                        P.BF16, ws)
    _assert_same_rounding(h.bits(y), ref, f"linear on few rows {M}x{K}x{N}")
    _counters_back_at_zero(ws)
    if res != "inplace":    # the same workspace serves the next call: bit-identical result
        y1 = torch.zeros_like(y)
        P.dllava_linear_few(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), torch.from_numpy(b).to(h.DEV), N, act, rd, y1,
                            N, P.BF16, ws)
        assert torch.equal(y1.view(torch.int16), y.view(torch.int16))
    # the tile kernel computes the same layer: the two agree to the rounding of the output
    y2 = torch.zeros((M, N), dtype=torch.bfloat16, device=h.DEV)
    if res == "inplace":
        y2.copy_(h.to_dev(r, "bf16"))
    P.dllava_linear(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), torch.from_numpy(b).to(h.DEV), N, act,
                    y2 if res == "inplace" else rd, y2, N, P.BF16)
    if K <= 11008:
        _assert_same_rounding(h.bits(y2), ref, "the tile kernel on the same rows")
    else:   # one float32 accumulator over a longer row of products: its error is no longer far below a step of the result
        assert (np.abs(R.widen(h.bits(y2), "bf16") - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-5).all()


def _few_workspace(nbytes: int, fill: int):
    """Workspace of a few-rows layer: zero-filled once where its counters live (the first 4096 bytes), junk elsewhere."""
    ws = torch.full((nbytes,), fill, dtype=torch.uint8, device=_H().DEV)
    ws[:4096] = 0
    return ws


def _counters_back_at_zero(ws):
    assert int(ws[:4096].to(torch.int32).sum().item()) == 0, "the counters of the workspace return to zero"


def test_rope_in_place():
    h = _H()
    rows, H, Dh = 37, 3, 128
    x = W.store(rng.normal(8, "x", (rows, H, Dh)), "bf16")
    pos = (rng.uniform01(8, "p", 0, rows) * 5000).astype(np.int32)
    ref = R.rope_rotate(R.widen(x, "bf16"), pos, DR.ROPE_BASE)
    xd = h.to_dev(x, "bf16")
    P.dllava_rope(xd, torch.from_numpy(pos).to(h.DEV), rows, H, Dh, DR.ROPE_BASE, P.BF16)
    _assert_same_rounding(h.bits(xd), ref, "rope")


@pytest.mark.parametrize("d,H,Dh,dff,n_layers,l,T", [(256, 2, 128, 512, 3, 1, 5), (4096, 32, 128, 11008, 1, 0, 2)],
                         ids=["three small layers", "one layer of the 7B shape"])
def test_decode_steps_through_the_stack(d, H, Dh, dff, n_layers, l, T):
    """Prefill with the reduction after layer l, then generated tokens one by one through all layers: the text
    predictor decides once per token (after layer l), layers before l keep every token, later layers the kept ones.
    (l = 0: the reduction and the decisions come before the first layer.)"""
    from paper_2412_00876_amd.layers import DecoderStack
    h = _H()
    w = W.make("stackd", "bf16", d, H, Dh, 3, [2, 0, 1], [40, 9, 70], [6, 3, 9], 0.3, T, seed=611)
    layers = W.decoder_layers(w, n_layers, dff)
    pred, predt = W.predictor(w), W.predictor(w, random_bias=True)
    x0 = W.store(rng.normal(w.seed, "h0", (w.sumN, d)), "bf16")
    xs = [W.store(rng.normal(w.seed, f"new{t}", (w.B, d)), "bf16") for t in range(T)]
    img = lambda rows: R.score(rows, pred["W1"], pred["b1"], pred["W2"], pred["b2"], "bf16")
    txt = lambda rows: R.score(rows, predt["W1"], predt["b1"], predt["W2"], predt["b2"], "bf16")
    n0 = np.diff(w.seq_off)
    cap = int(n0.max()) + T
    mp = (cap + 15) // 16
    caches = [R.PagedCache(w.B * mp, np.arange(w.B * mp, dtype=np.int32).reshape(w.B, mp), H, Dh, "bf16") for _ in layers]
    xf, idx, off, _ = DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, l, w.keep_ratio, img, H, Dh, "bf16",
                                         True, caches)
    M_vis = int(sum(w.n_vis))
    S = DecoderStack(_upload_layers(h, layers), l, w.B, H, Dh, d, dff, w.sumN, M_vis, max_seq_len=int(n0.max()), extra_tokens=T)
    i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).to(h.DEV)
    seq_off, vis_start, vis_len = i32(w.seq_off), i32(w.vis_start), i32(w.vis_len)
    up = lambda P_: {k: (h.to_dev(v, "bf16") if v.dtype == np.uint16 else torch.from_numpy(v).to(h.DEV)) for k, v in P_.items()}
    pw, pt = up(pred), up(predt)
    ws = torch.zeros(P.dllava_score_workspace(max(M_vis, 64), d, w.dh, P.BF16), dtype=torch.uint8, device=h.DEV)

    def image_predictor(X, logits):
        P.dllava_score(X, d, M_vis, w.B, seq_off, vis_start, vis_len, d, w.dh, pw["W1"], pw["b1"], pw["W2"], pw["b2"], P.BF16,
                       logits, ws)

    def text_predictor(X, logits):
        P.dllava_score(X, d, w.B, 0, None, None, None, d, w.dh, pt["W1"], pt["b1"], pt["W2"], pt["b2"], P.BF16, logits, ws)

    S.prefill(h.to_dev(x0, "bf16"), seq_off, vis_start, vis_len, w.keep_ratio, int(off[-1]), image_predictor)
    assert np.array_equal(S.out_off.cpu().numpy(), off)
    theta = 0.0
    for t in range(T):
        pos = n0 + t
        xo_ref, keep_ref, logits_ref = DR.decoder_decode_step(xs[t], pos, layers, caches, l, theta, txt, H, Dh, "bf16")
        xo = S.decode_step(h.to_dev(xs[t], "bf16"), i32(pos), theta, text_predictor)
        torch.cuda.synchronize()
        lg = S.logits_d.cpu().numpy()
        assert np.abs(lg - logits_ref).max() <= 5e-2
        assert np.abs((logits_ref[:, 1] - logits_ref[:, 0]) - theta).min() > 4 * np.abs(lg - logits_ref).max()   # away from ties
        assert np.array_equal(S.keep_d.cpu().numpy(), keep_ref)
        err = h.as_f64(xo) - xo_ref
        scale = np.sqrt(np.mean(xo_ref ** 2))
        assert np.sqrt(np.mean(err ** 2)) <= 2e-2 * scale and np.abs(err).max() <= 0.15 * scale, t
        for i in range(n_layers):
            assert np.array_equal(S.caches[i].cache_len.cpu().numpy(), caches[i].cache_len), (t, i)
    assert int(S.err.item()) == 0
    if l > 0:
        assert list(caches[0].cache_len) == list(n0 + T)                             # a layer before l keeps every token
    if n_layers > 2:
        assert list(caches[2].cache_len) != list(np.diff(off) + T)                   # later layers dropped some


@pytest.mark.parametrize("M,d,H,Dh", [(16, 4096, 32, 128), (5, 256, 2, 64), (40, 320, 3, 32), (32, 5120, 40, 128), (1, 4096, 32, 128)])
def test_fused_qkv_of_a_decode_step(M, d, H, Dh):
    h = _H()
    seed = 4000 + M + d
    x = W.store(rng.normal(seed, "x", (M, d)), "bf16")
    Ws = [W.store(W._normal_big(seed, n, (H * Dh, d)) / np.sqrt(d), "bf16") for n in "qkv"]
    pos = (rng.uniform01(seed, "p", 0, M) * 3000).astype(np.int32)
    xs = R.widen(x, "bf16")
    q, k, v = ((xs @ R.widen(Wm, "bf16").T).reshape(M, H, Dh) for Wm in Ws)
    q, k = R.rope_rotate(q, pos, DR.ROPE_BASE), R.rope_rotate(k, pos, DR.ROPE_BASE)
    out = [torch.zeros((M, H, Dh), dtype=torch.bfloat16, device=h.DEV) for _ in range(3)]
    ws = _few_workspace(P.dllava_decode_proj_workspace(3 * H * Dh, d), 0x21)
    for _ in range(2):      # the second call finds the workspace as the first one left it
        for o in out:
            o.zero_()
        P.dllava_qkv_few(h.to_dev(x, "bf16"), d, M, d, *(h.to_dev(Wm, "bf16") for Wm in Ws), H, Dh,
                         torch.from_numpy(pos).to(h.DEV), DR.ROPE_BASE, *out, P.BF16, ws)
        for got, ref, name in zip(out, (q, k, v), "qkv"):
            _assert_same_rounding(h.bits(got), ref, f"fused {name}")
        _counters_back_at_zero(ws)


@pytest.mark.parametrize("M,d,F", [(16, 4096, 11008), (3, 128, 96), (37, 512, 64), (32, 5120, 13824), (1, 4096, 11008)])
def test_fused_gated_layer_of_a_decode_step(M, d, F):
    h = _H()
    seed = 5000 + M + d
    x = W.store(rng.normal(seed, "x", (M, d)), "bf16")
    Wg = W.store(W._normal_big(seed, "g", (F, d)) / np.sqrt(d) * 2, "bf16")
    Wu = W.store(W._normal_big(seed, "u", (F, d)) / np.sqrt(d), "bf16")
    xs = R.widen(x, "bf16")
    gate = R.widen(R.narrow(xs @ R.widen(Wg, "bf16").T, "bf16"), "bf16")          # the gate as if it had been stored
    ref = DR.silu(gate) * (xs @ R.widen(Wu, "bf16").T)
    y = torch.zeros((M, F), dtype=torch.bfloat16, device=h.DEV)
    ws = _few_workspace(P.dllava_decode_proj_workspace(2 * F, d), 0x21)
    P.dllava_gated_few(h.to_dev(x, "bf16"), d, M, d, h.to_dev(Wg, "bf16"), h.to_dev(Wu, "bf16"), F, y, F, P.BF16, ws)
    _counters_back_at_zero(ws)
    # where the GPU's float32 gate sum rounds to the other neighbour, the product moves by the gate's step times the
    # slope of SiLU: allowed as a one-step difference of the gate, counted with the other one-step differences
    got = R.widen(h.bits(y), "bf16")
    err = np.abs(got - ref)
    up = np.abs(xs @ R.widen(Wu, "bf16").T)
    assert (err <= 2.0 ** -7 * np.abs(ref) + 1.2 * 2.0 ** -8 * np.abs(gate) * up + 1e-6).all()
    assert (h.bits(y) != R.narrow(ref, "bf16")).mean() <= 0.03


def test_few_rows_layers_replay_from_a_hip_graph():
    """RMSNorm -> q|k|v -> W_O with residual -> gate|up -> down-projection on few rows, with shapes whose blocks hand
    sums over through the workspace counters, captured once and replayed: every replay reproduces the eager result
    bit for bit and leaves the counters at zero."""
    h = _H()
    M, d, H, Dh, F, wide = 9, 512, 4, 32, 64, 2048
    HD = H * Dh
    dev = lambda name, shape, s=1.0: h.to_dev(W.store(W._normal_big(77, name, shape) * s, "bf16"), "bf16")
    x = dev("x", (M, d))
    Wq, Wk, Wv = (dev(n, (HD, d), d ** -0.5) for n in "qkv")
    Wo, Wg, Wu, Wd = dev("o", (d, HD), HD ** -0.5), dev("g", (F, d), d ** -0.5), dev("u", (F, d), d ** -0.5), dev("d", (d, F), F ** -0.5)
    Ww, xw = dev("w", (64, wide), wide ** -0.5), dev("xw", (M, wide))
    gam = torch.from_numpy(rng.uniform(77, "gam", (d,), 0.5, 1.5).astype(np.float32)).to(h.DEV)
    pos = torch.arange(100, 100 + M, dtype=torch.int32, device=h.DEV)
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device=h.DEV)
    y, q, k, v, x1, f, x2, yw = z(M, d), z(M, H, Dh), z(M, H, Dh), z(M, H, Dh), z(M, d), z(M, F), z(M, d), z(M, 64)
    ws = _few_workspace(max(P.dllava_decode_proj_workspace(3 * HD, d), P.dllava_decode_proj_workspace(2 * F, d),
                            P.dllava_linear_few_workspace(d, HD), P.dllava_linear_few_workspace(d, F),
                            P.dllava_linear_few_workspace(64, wide)), 0x5a)

    def chain():
        P.dllava_rms_norm(x, d, M, d, gam, 1e-5, y, d, P.BF16)
        P.dllava_qkv_few(y, d, M, d, Wq, Wk, Wv, H, Dh, pos, 10000.0, q, k, v, P.BF16, ws)
        P.dllava_linear_few(q, HD, M, HD, Wo, None, d, 0, x, x1, d, P.BF16, ws)
        P.dllava_gated_few(x1, d, M, d, Wg, Wu, F, f, F, P.BF16, ws)
        P.dllava_linear_few(f, F, M, F, Wd, None, d, 0, x1, x2, d, P.BF16, ws)
        P.dllava_linear_few(xw, wide, M, wide, Ww, None, 64, 1, None, yw, 64, P.BF16, ws)

    outs = (y, q, k, v, x1, f, x2, yw)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        chain()
        st.synchronize()
        ref = [t.clone() for t in outs]
        assert all(bool(t.float().abs().sum() > 0) for t in ref)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            chain()
        for rep in range(3):
            for t in outs:
                t.zero_()                                      # eager work between replays
            ws[4096:].fill_(rep + 1)
            st.synchronize()
            graph.replay()
            st.synchronize()
            for i, (a, b) in enumerate(zip(ref, outs)):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (rep, i)
            _counters_back_at_zero(ws)


@pytest.mark.parametrize("M,K,N", [(7, 512, 4096), (20, 2048, 64), (40, 4096, 12288)])
def test_few_rows_layers_with_padded_rows(M, K, N):
    """Input rows with a stride larger than K and output / residual rows with a stride larger than N: the padding is
    neither read into the result nor written."""
    h = _H()
    seed = 7000 + M + K + N
    ldx, ldy = K + 64, N + 40
    x = W.store(rng.normal(seed, "x", (M, K)), "bf16")
    Wm = W.store(W._normal_big(seed, "W", (N, K)) / np.sqrt(K), "bf16")
    r = W.store(rng.normal(seed, "r", (M, N)), "bf16")
    ref = R.widen(x, "bf16") @ R.widen(Wm, "bf16").T + R.widen(r, "bf16")
    xp = torch.full((M, ldx), float("nan"), dtype=torch.bfloat16, device=h.DEV)
    xp[:, :K] = h.to_dev(x, "bf16")
    rp = torch.full((M, ldy), float("nan"), dtype=torch.bfloat16, device=h.DEV)
    rp[:, :N] = h.to_dev(r, "bf16")
    y = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device=h.DEV)
    ws = _few_workspace(P.dllava_linear_few_workspace(N, K), 0x11)
    P.dllava_linear_few(xp, ldx, M, K, h.to_dev(Wm, "bf16"), None, N, 0, rp, y, ldy, P.BF16, ws)
    got = h.bits(y)
    _assert_same_rounding(got[:, :N], ref, f"padded rows {M}x{K}x{N}")
    assert bool((y[:, N:] == 7.0).all()), "columns past N are left alone"
    _counters_back_at_zero(ws)
    if N % 3 == 0 and (N // 3) % 32 == 0:        # the same input through the fused q|k|v layer (rotation at position 0: none)
        H, Dh = N // 3 // 32, 32
        outs = [torch.zeros((M, H, Dh), dtype=torch.bfloat16, device=h.DEV) for _ in range(3)]
        Wd = h.to_dev(Wm, "bf16")
        ws2 = _few_workspace(P.dllava_decode_proj_workspace(N, K), 0x12)
        P.dllava_qkv_few(xp, ldx, M, K, Wd[:N // 3], Wd[N // 3:2 * N // 3], Wd[2 * N // 3:], H, Dh,
                         torch.zeros(M, dtype=torch.int32, device=h.DEV), 10000.0, *outs, P.BF16, ws2)
        plain = R.widen(x, "bf16") @ R.widen(Wm, "bf16").T
        for i, o in enumerate(outs):
            _assert_same_rounding(h.bits(o).reshape(M, -1), plain[:, i * N // 3:(i + 1) * N // 3], f"q|k|v part {i} from padded rows")


@pytest.mark.parametrize("seed", range(12))
def test_few_rows_layers_on_random_shapes(seed):
    """Seeded random shapes through the three few-rows entry points (all block shapes and hand-over paths are reached
    over the seeds), each against the float64 product to the rounding of its output."""
    h = _H()
    u = lambda name, lo, hi: int(lo + rng.uniform01(9000 + seed, name, 0, 1)[0] * (hi - lo + 0.999))
    M = [1, 3, 16, 17, 32, 33, 50, 64][u("M", 0, 7)]
    K = 64 * u("K", 1, 40)
    N = 32 * u("N", 1, 48)
    x = W.store(rng.normal(seed, "x", (M, K)), "bf16")
    xs = R.widen(x, "bf16")
    Wm = W.store(W._normal_big(seed, "W", (N, K)) / np.sqrt(K), "bf16")
    b = rng.uniform(seed, "b", (N,), -0.5, 0.5).astype(np.float32)
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=h.DEV)
    ws = _few_workspace(P.dllava_linear_few_workspace(N, K), 0x3c)
    P.dllava_linear_few(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), torch.from_numpy(b).to(h.DEV), N, 1, None, y, N,
                        P.BF16, ws)
    _assert_same_rounding(h.bits(y), R.gelu(xs @ R.widen(Wm, "bf16").T + b), f"linear {M}x{K}x{N}")
    _counters_back_at_zero(ws)
    # gate|up with F = N and q|k|v with H heads of 32 or 64 (H * Dh = N when that divides)
    Wu = W.store(W._normal_big(seed, "U", (N, K)) / np.sqrt(K), "bf16")
    f = torch.zeros((M, N), dtype=torch.bfloat16, device=h.DEV)
    ws2 = _few_workspace(P.dllava_decode_proj_workspace(2 * N, K), 0x3d)
    P.dllava_gated_few(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), h.to_dev(Wu, "bf16"), N, f, N, P.BF16, ws2)
    gate = R.widen(R.narrow(xs @ R.widen(Wm, "bf16").T, "bf16"), "bf16")
    up = xs @ R.widen(Wu, "bf16").T
    ref = DR.silu(gate) * up
    err = np.abs(R.widen(h.bits(f), "bf16") - ref)
    assert (err <= 2.0 ** -7 * np.abs(ref) + 1.2 * 2.0 ** -8 * np.abs(gate) * np.abs(up) + 1e-6).all()
    _counters_back_at_zero(ws2)
    Dh = 64 if N % 64 == 0 and seed % 2 else 32
    H = N // Dh
    pos = (rng.uniform01(seed, "p", 0, M) * 4000).astype(np.int32)
    outs = [torch.zeros((M, H, Dh), dtype=torch.bfloat16, device=h.DEV) for _ in range(3)]
    Wv = W.store(W._normal_big(seed, "V", (N, K)) / np.sqrt(K), "bf16")
    ws3 = _few_workspace(P.dllava_decode_proj_workspace(3 * N, K), 0x3e)
    P.dllava_qkv_few(h.to_dev(x, "bf16"), K, M, K, h.to_dev(Wm, "bf16"), h.to_dev(Wu, "bf16"), h.to_dev(Wv, "bf16"), H, Dh,
                     torch.from_numpy(pos).to(h.DEV), DR.ROPE_BASE, *outs, P.BF16, ws3)
    q, k, v = ((xs @ R.widen(m_, "bf16").T).reshape(M, H, Dh) for m_ in (Wm, Wu, Wv))
    q, k = R.rope_rotate(q, pos, DR.ROPE_BASE), R.rope_rotate(k, pos, DR.ROPE_BASE)
    for got, want, name in zip(outs, (q, k, v), "qkv"):
        _assert_same_rounding(h.bits(got), want, f"fused {name} {M}x{K}x{N}")
    _counters_back_at_zero(ws3)
