"""Pins for the CPU oracle: values the paper prints, closed forms, brute force on tiny inputs.

Each check is written independently of oracle/dllava_ref.py (pure-Python loops, a different
formulation of the same definition, or a printed number), so that a dropped term, a wrong sign or
index, or a transposed operand in the oracle fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

from oracle import dllava_ref as R
from synth import workloads as W
from synth import rng

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ------------------------------------------------------------------ printed numbers (Table 1, Eq. 11, Eq. 13)

def test_keep_count_matches_printed_token_counts():
    for n, r, k in _rows("keep_counts.txt"):
        assert R.keep_count(float(r), int(n)) == int(k)


def test_eq13_reproduces_table1_tflops():
    for model, C, L, method, after, tokens, printed in _rows("table1_image_prefill.txt"):
        got = R.model_prefill_tflops(576, int(tokens), int(C), int(L), int(after))
        assert abs(got - float(printed)) <= 0.05 + 1e-9, (model, method, got, printed)
    # the printed 2.5 / 4.7 need BOTH l = 2 dense layers and k = 115: neighbours miss the rounding window
    assert round(R.model_prefill_tflops(576, 115, 4096, 32, 2), 1) == 2.5
    assert round(R.model_prefill_tflops(576, 115, 4096, 32, 0), 1) != 2.5
    assert round(R.model_prefill_tflops(576, 115, 5120, 40, 2), 1) == 4.7
    assert round(R.model_prefill_tflops(576, 115, 5120, 40, 4), 1) != 4.7


# ------------------------------------------------------------------ predictor

def _score_loops(x, W1, b1, W2, b2):
    M, d = x.shape
    dh = W1.shape[0]
    D = np.zeros((M, 2))
    for i in range(M):
        h = []
        for j in range(dh):
            a = float(b1[j])
            for c in range(d):
                a += float(x[i, c]) * float(W1[j, c])
            h.append(0.5 * a * (1.0 + math.erf(a / math.sqrt(2.0))))
        for o in range(2):
            D[i, o] = float(b2[o]) + sum(h[j] * float(W2[o, j]) for j in range(dh))
    return D


def test_gelu_closed_form_values():
    # GELU(a) = a * Phi(a); Phi(1) = 0.8413447460685429, Phi(-1) = 1 - Phi(1), Phi(2) = 0.9772498680518208
    a = np.array([0.0, 1.0, -1.0, 2.0, 40.0, -40.0])
    g = R.gelu(a)
    exp = [0.0, 0.8413447460685429, -(1 - 0.8413447460685429), 2 * 0.9772498680518208, 40.0, 0.0]
    assert np.allclose(g, exp, rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_vs_triple_loop(dtype):
    M, d, dh = 5, 12, 7
    x = W.store(rng.normal(11, "x", (M, d)), dtype)
    W1 = W.store(rng.normal(11, "W1", (dh, d)) * 0.5, dtype)
    W2 = W.store(rng.normal(11, "W2", (2, dh)), dtype)
    b1 = rng.normal(11, "b1", (dh,))
    b2 = rng.normal(11, "b2", (2,))
    ref = _score_loops(W.stored_to_f32(x, dtype), W.stored_to_f32(W1, dtype), b1,
                       W.stored_to_f32(W2, dtype), b2)
    got = R.score(x, W1, b1, W2, b2, dtype)
    assert got.dtype == np.float32 and got.shape == (M, 2)
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    # columns are not interchangeable and W1 is used as [dh, d] (not transposed)
    assert not np.allclose(got[:, 0], got[:, 1])


def test_score_special_cases():
    M, d, dh = 4, 8, 6
    x = rng.normal(3, "x", (M, d))
    W2 = rng.normal(3, "W2", (2, dh))
    b1 = rng.normal(3, "b1", (dh,))
    b2 = np.array([0.25, -0.5], np.float32)
    # zero first layer: D = b2 + GELU(b1) W2^T for every row
    D = R.score(x, np.zeros((dh, d), np.float32), b1, W2, b2, "f32")
    g = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in b1.astype(np.float64)])
    exp = b2.astype(np.float64) + W2.astype(np.float64) @ g
    assert np.allclose(D, np.tile(exp, (M, 1)), atol=1e-6)
    # W2 = [0; e_j] picks hidden unit j into the keep column, nothing into the drop column
    W1 = rng.normal(3, "W1", (dh, d))
    E = np.zeros((2, dh), np.float32)
    E[1, 2] = 1.0
    D = R.score(x, W1, None, E, None, "f32")
    a = x.astype(np.float64) @ W1.astype(np.float64)[2]
    assert np.allclose(D[:, 0], 0.0)
    assert np.allclose(D[:, 1], [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in a], atol=1e-6)


# ------------------------------------------------------------------ selection

def _topk_rank_count(s, k):
    """Definition by counting: token i is kept iff fewer than k tokens beat it."""
    n = len(s)

    def beats(j, i):           # j ranks strictly ahead of i
        a, b = float(s[j]), float(s[i])
        an, bn = a != a, b != b
        if an or bn:
            if an and bn:
                return j < i
            return bn          # a number beats NaN
        if a != b:
            return a > b
        return j < i
    return np.array([i for i in range(n) if sum(beats(j, i) for j in range(n) if j != i) < k], np.int32)


@pytest.mark.parametrize("seed", range(6))
def test_topk_equals_rank_count_with_ties(seed):
    n = 37
    s = rng.normal(seed, "s", (n,))
    s = np.round(s * 2) / 2            # many exact ties
    s[3] = 0.0
    s[9] = -0.0
    if seed % 2:
        s[5] = np.nan
        s[20] = np.nan
        s[7] = np.inf
        s[8] = -np.inf
    for k in (0, 1, 5, 17, n - 1, n, n + 3):
        got = R.select_topk(s, k)
        exp = _topk_rank_count(s, min(k, n))
        assert np.array_equal(got, exp), (seed, k)
        assert len(got) == min(k, n) and np.all(np.diff(got) > 0)


def test_topk_tie_goes_to_lower_index():
    s = np.array([1.0, 2.0, 2.0, 2.0, 0.5], np.float32)
    assert list(R.select_topk(s, 2)) == [1, 2]
    assert list(R.select_topk(np.array([0.0, -0.0, 0.0], np.float32), 2)) == [0, 1]


def test_threshold_is_strict_argmax_rule():
    D = np.array([[0.0, 1.0], [1.0, 0.0], [0.5, 0.5], [-1.0, -0.5]], np.float32)
    assert list(R.select_threshold(D, 0.0)) == [1, 0, 0, 1]          # tie -> drop (Eq. 5: "greater than")
    assert list(R.select_threshold(D, -np.inf)) == [1, 1, 1, 1]
    assert list(R.select_threshold(D, np.inf)) == [0, 0, 0, 0]
    assert list(R.select_threshold(D, 0.5)) == [1, 0, 0, 0]


def _ragged():
    return W.make("ragged", "bf16", 32, 2, 16, 3, [3, 0, 5], [20, 33, 7], [4, 9, 0], 0.3, 6)


def test_select_counts_and_order():
    w = _ragged()
    D = rng.normal(5, "D", (int(sum(w.n_vis)), 2))
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    for b in range(w.B):
        s0, s1 = w.seq_off[b], w.seq_off[b + 1]
        k = math.floor(w.keep_ratio * w.n_vis[b])
        assert off[b + 1] - off[b] == int(mask[s0:s1].sum()) == w.n_sys[b] + k + w.n_prompt[b]
        ib = idx[off[b]:off[b + 1]]
        assert np.all(np.diff(ib) > 0) and np.all(mask[s0 + ib] == 1)
        # text rows all kept
        assert mask[s0:s0 + w.n_sys[b]].all() and mask[s0 + w.n_sys[b] + w.n_vis[b]:s1].all()
    # keep everything / nothing
    m1, i1, o1 = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, 1.0, 0.0)
    assert m1.all() and list(o1) == list(w.seq_off)
    m0, i0, o0 = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, 0.0, 0.0)
    assert int(m0.sum()) == sum(w.n_sys) + sum(w.n_prompt)


# ------------------------------------------------------------------ attention, brute force

def _attn_row_loops(q, keys, vals, scale):
    """softmax(scale * q.k_j) weighted mean of v_j, pure Python, float64."""
    s = [scale * sum(float(a) * float(b) for a, b in zip(q, k)) for k in keys]
    m = max(s)
    p = [math.exp(v - m) for v in s]
    z = sum(p)
    return [sum(p[j] * float(vals[j][c]) for j in range(len(keys))) / z for c in range(len(vals[0]))]


def _tiny(dtype="bf16", T=5, ratio=0.4):
    w = W.make("tiny", dtype, 16, 2, 8, 2, [2, 1], [9, 6], [3, 2], ratio, T)
    pre = W.prefill_inputs(w)
    dec = W.decode_inputs(w)
    return w, pre, dec


def _run_oracle(w, pre, dec, ratio, theta, D=None, keep_seq=None):
    if D is None:
        D = rng.normal(w.seed, "pins.D", (int(sum(w.n_vis)), 2))
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, ratio, 0.0)
    bt, n_pages = W.block_table(w, extra_tokens=max(w.seq_len))
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    _, Qc = R.compact(idx, off, w.seq_off, hidden=None, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    Kc = np.concatenate([cache.rows(b)[0] for b in range(w.B)])
    Vc = np.concatenate([cache.rows(b)[1] for b in range(w.B)])
    scale = 1.0 / math.sqrt(w.Dh)
    O = R.prefill_attn(Qc, Kc, Vc, off, scale, w.dtype)
    outs, keeps = [], []
    Dt = rng.normal(w.seed, "pins.Dt", (w.T, w.B, 2))
    for t in range(w.T):
        keep = R.decode_keep(Dt[t], theta) if keep_seq is None else keep_seq[t]
        o, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep, cache, scale)
        assert not err.any()
        outs.append(o)
        keeps.append(np.array(keep))
    return mask, idx, off, O, outs, keeps, cache


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_keep_everything_is_dense_causal_attention(dtype):
    """ratio 1.0 and threshold -inf: prefill and every decode step equal dense attention over all tokens."""
    w, pre, dec = _tiny(dtype)
    mask, idx, off, O, outs, keeps, cache = _run_oracle(w, pre, dec, 1.0, -np.inf)
    assert mask.all() and all(k.all() for k in keeps)
    f = lambda a: W.stored_to_f32(a, dtype).astype(np.float64)
    Q, K, V = f(pre["Q"]), f(pre["K"]), f(pre["V"])
    scale = 1.0 / math.sqrt(w.Dh)
    for b in range(w.B):
        s0, s1 = int(w.seq_off[b]), int(w.seq_off[b + 1])
        for h in range(w.H):
            for i in range(s0, s1):
                ref = _attn_row_loops(Q[i, h], K[s0:i + 1, h], V[s0:i + 1, h], scale)
                assert np.allclose(O[i, h], ref, atol=1e-12)
            for t in range(w.T):
                keys = list(K[s0:s1, h]) + [f(dec["k"][u])[b, h] for u in range(t + 1)]
                vals = list(V[s0:s1, h]) + [f(dec["v"][u])[b, h] for u in range(t + 1)]
                ref = _attn_row_loops(f(dec["q"][t])[b, h], keys, vals, scale)
                assert np.allclose(outs[t][b, h], ref, atol=1e-12)
    assert list(cache.cache_len) == [n + w.T for n in w.seq_len]


def _masked_softmax_attention(Q, K, V, M, scale):
    """Eq. 7 with a causal mask: dense N x N attention, G[i,j] = M[j], diag(G) = 1.  Returns [N,Dh]."""
    N = len(Q)
    out = np.zeros((N, V.shape[1]))
    for i in range(N):
        x = [scale * float(Q[i] @ K[j]) for j in range(i + 1)]
        g = [1.0 if (j == i or M[j]) else 0.0 for j in range(i + 1)]
        mx = max(x)
        e = [math.exp(x[j] - mx) * g[j] for j in range(i + 1)]
        z = sum(e)
        for j in range(i + 1):
            out[i] += (e[j] / z) * V[j]
    return out


def test_gather_form_equals_masked_softmax_form():
    """Inference (gather then causal attention) == training form (Eq. 7 mask on the full sequence),
    for prefill rows that are kept and for every decode step under an arbitrary keep history."""
    w, pre, dec = _tiny("bf16", T=6, ratio=0.4)
    keep_seq = [np.array(v, np.uint8) for v in ([1, 0], [0, 0], [1, 1], [0, 1], [1, 0], [0, 1])]
    mask, idx, off, O, outs, keeps, cache = _run_oracle(w, pre, dec, 0.4, 0.0, keep_seq=keep_seq)
    f = lambda a: W.stored_to_f32(a, "bf16").astype(np.float64)
    scale = 1.0 / math.sqrt(w.Dh)
    for b in range(w.B):
        s0, s1 = int(w.seq_off[b]), int(w.seq_off[b + 1])
        Mfull = list(mask[s0:s1]) + [int(keep_seq[t][b]) for t in range(w.T)]
        for h in range(w.H):
            Qa = np.concatenate([f(pre["Q"])[s0:s1, h], np.stack([f(dec["q"][t])[b, h] for t in range(w.T)])])
            Ka = np.concatenate([f(pre["K"])[s0:s1, h], np.stack([f(dec["k"][t])[b, h] for t in range(w.T)])])
            Va = np.concatenate([f(pre["V"])[s0:s1, h], np.stack([f(dec["v"][t])[b, h] for t in range(w.T)])])
            dense = _masked_softmax_attention(Qa, Ka, Va, Mfull, scale)
            kept_rows = idx[off[b]:off[b + 1]]
            assert np.allclose(O[off[b]:off[b + 1], h], dense[kept_rows], atol=1e-12)
            for t in range(w.T):
                assert np.allclose(outs[t][b, h], dense[(s1 - s0) + t], atol=1e-12)
    exp_len = [int(off[b + 1] - off[b]) + sum(int(k[b]) for k in keep_seq) for b in range(w.B)]
    assert list(cache.cache_len) == exp_len


def test_masked_attn_matches_loops_and_its_special_cases():
    """R.masked_attn (Eq. 7 on the full token set) against the loop form above, and: all-ones mask = causal attention,
    all-zeros mask = every row returns its own value, kept rows = attention over the compacted sequence, a dropped
    token influences no row but its own."""
    w, pre, dec = _tiny("bf16", T=1, ratio=0.4)
    f = lambda a: W.stored_to_f32(a, "bf16").astype(np.float64)
    scale = 1.0 / math.sqrt(w.Dh)
    r = np.random.RandomState(3)
    keep = (r.rand(w.sumN) < 0.5).astype(np.uint8)
    O = R.masked_attn(pre["Q"], pre["K"], pre["V"], w.seq_off, keep, scale, "bf16")
    for b in range(w.B):
        s0, s1 = int(w.seq_off[b]), int(w.seq_off[b + 1])
        for h in range(w.H):
            dense = _masked_softmax_attention(f(pre["Q"])[s0:s1, h], f(pre["K"])[s0:s1, h], f(pre["V"])[s0:s1, h],
                                              list(keep[s0:s1]), scale)
            assert np.allclose(O[s0:s1, h], dense, atol=1e-12)
    ones = R.masked_attn(pre["Q"], pre["K"], pre["V"], w.seq_off, np.ones(w.sumN, np.uint8), scale, "bf16")
    assert np.allclose(ones, R.prefill_attn(pre["Q"], pre["K"], pre["V"], w.seq_off, scale, "bf16"), atol=1e-12)
    zeros = R.masked_attn(pre["Q"], pre["K"], pre["V"], w.seq_off, np.zeros(w.sumN, np.uint8), scale, "bf16")
    assert np.allclose(zeros, f(pre["V"]), atol=1e-12)
    # kept rows: the compacted sequence attended causally
    idx = np.flatnonzero(keep)
    off_c = np.concatenate([[0], np.cumsum([keep[w.seq_off[b]:w.seq_off[b + 1]].sum() for b in range(w.B)])])
    Oc = R.prefill_attn(pre["Q"][idx], pre["K"][idx], pre["V"][idx], off_c, scale, "bf16")
    assert np.allclose(O[idx], Oc, atol=1e-12)
    # the row-by-row form used for long sequences
    some = [0, 1, int(w.seq_off[1]) - 1, int(w.seq_off[1]), w.sumN - 1]
    assert np.allclose(R.masked_attn_rows(pre["Q"], pre["K"], pre["V"], w.seq_off, keep, scale, "bf16", some), O[some],
                       atol=1e-12)
    # a dropped token's key and value matter to its own row only
    j = int(np.flatnonzero(keep == 0)[1])
    K2, V2 = pre["K"].copy(), pre["V"].copy()
    K2[j], V2[j] = pre["K"][j - 1], pre["V"][j - 1]
    O2 = R.masked_attn(pre["Q"], K2, V2, w.seq_off, keep, scale, "bf16")
    others = np.arange(w.sumN) != j
    assert np.array_equal(O2[others], O[others]) and not np.allclose(O2[j], O[j])


def test_decode_closed_forms():
    H, Dh = 2, 8
    bt = np.array([[1, 0]], np.int32)
    cache = R.PagedCache(2, bt, H, Dh, "f32", page_size=4)
    q = rng.normal(1, "q", (1, H, Dh))
    k = rng.normal(1, "k", (1, H, Dh))
    v = rng.normal(1, "v", (1, H, Dh))
    # empty cache: softmax over the single (current) key is 1 -> o == v_new; token not kept -> cache stays empty
    o, _ = R.decode_attn_append(q, k, v, [0], cache, 0.3)
    assert np.array_equal(o.astype(np.float32), v) and cache.cache_len[0] == 0
    # identical keys: uniform weights -> arithmetic mean of the values (cached ones and the new one)
    vs = [rng.normal(2, f"v{t}", (1, H, Dh)) for t in range(6)]
    for t in range(5):
        R.decode_attn_append(q, k, vs[t], [1], cache, 0.3)
    assert cache.cache_len[0] == 5
    o, _ = R.decode_attn_append(q, k, vs[5], [0], cache, 0.3)
    assert np.allclose(o, np.mean([a.astype(np.float64) for a in vs], axis=0), atol=1e-12)
    # a key aligned with q with a huge logit takes all the weight
    kbig = (q * 1000).astype(np.float32)
    vbig = rng.normal(3, "vbig", (1, H, Dh))
    o, _ = R.decode_attn_append(q, kbig, vbig, [0], cache, 1.0)
    assert np.allclose(o, vbig, atol=1e-9)
    # capacity: 8 slots; fill up, then a kept token is flagged and not stored
    for t in range(3):
        _, err = R.decode_attn_append(q, k, v, [1], cache, 0.3)
        assert not err.any()
    assert cache.cache_len[0] == 8
    _, err = R.decode_attn_append(q, k, v, [1], cache, 0.3)
    assert err[0] == 1 and cache.cache_len[0] == 8


def test_outputs_are_convex_combinations_and_page_placement_is_irrelevant():
    w, pre, dec = _tiny("bf16", T=4, ratio=0.5)
    a = _run_oracle(w, pre, dec, 0.5, 0.0)
    w2 = W.make("tiny", "bf16", 16, 2, 8, 2, [2, 1], [9, 6], [3, 2], 0.5, 4, seed=w.seed)
    O, outs, cache = a[3], a[4], a[6]
    # each output channel lies within the range of the values it averages
    f = lambda x: W.stored_to_f32(x, "bf16").astype(np.float64)
    for b in range(w.B):
        Kc, Vc = cache.rows(b)
        Vf = f(Vc)
        for h in range(w.H):
            lo = np.minimum(Vf[:, h].min(0), f(dec["v"][-1])[b, h])
            hi = np.maximum(Vf[:, h].max(0), f(dec["v"][-1])[b, h])
            assert np.all(outs[-1][b, h] >= lo - 1e-12) and np.all(outs[-1][b, h] <= hi + 1e-12)
    # a different block table (reversed page ids) gives bit-identical outputs
    mask, idx, off = a[0], a[1], a[2]
    bt, n_pages = W.block_table(w, extra_tokens=max(w.seq_len))
    cache2 = R.PagedCache(n_pages, (n_pages - 1 - bt), w.H, w.Dh, w.dtype)
    R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache2)
    scale = 1.0 / math.sqrt(w.Dh)
    for t in range(w.T):
        o2, _ = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], a[5][t], cache2, scale)
        assert np.array_equal(o2, outs[t])


def test_compact_copies_kept_rows_bit_exactly():
    w, pre, dec = _tiny("bf16")
    D = rng.normal(9, "D", (int(sum(w.n_vis)), 2))
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    bt, n_pages = W.block_table(w)
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    h_out, q_out = R.compact(idx, off, w.seq_off, hidden=pre["hidden"], Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    j = 0
    for b in range(w.B):
        Kc, Vc = cache.rows(b)
        for t, p in enumerate(idx[off[b]:off[b + 1]]):
            src = int(w.seq_off[b]) + int(p)
            assert np.array_equal(h_out[j], pre["hidden"][src]) and np.array_equal(q_out[j], pre["Q"][src])
            assert np.array_equal(Kc[t], pre["K"][src]) and np.array_equal(Vc[t], pre["V"][src])
            j += 1
    assert j == off[-1] == len(h_out)


# ------------------------------------------------------------------ projection of the reduced set (Eq. 3 line 1)

def test_narrow_rounds_to_nearest_even_and_inverts_widen():
    # 1 + 2^-8 lies exactly between two bfloat16 values: the even mantissa (1.0) wins; 1 + 3*2^-8 goes up to 1 + 2^-6
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20, 0.0, -0.0])
    got = R.widen(R.narrow(a, "bf16"), "bf16")
    assert np.array_equal(got, np.array([1.0, 1.0 + 2.0 ** -6, -1.0, 1.0 + 2.0 ** -7, 0.0, 0.0]))
    bits = np.arange(0, 0x7F80, 7, dtype=np.uint16)  # every 7th finite positive pattern
    assert np.array_equal(R.narrow(R.widen(bits, "bf16"), "bf16"), bits)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_projection_vs_triple_loop(dtype):
    rows, d, H, Dh = 5, 24, 2, 8
    x = W.store(rng.normal(5, "x", (rows, d)).astype(np.float32), dtype)
    Ws = [W.store(rng.normal(5, f"W{i}", (H * Dh, d)).astype(np.float32) * 0.3, dtype) for i in range(3)]
    Q, K, V = R.qkv_project(x, np.array([0, 2, 5]), np.zeros(rows, np.int64), *Ws, H, Dh, dtype)
    xf = [[float(v) for v in r] for r in W.stored_to_f32(x, dtype)]
    for got, Wm in zip((Q, K, V), Ws):
        wf = [[float(v) for v in r] for r in W.stored_to_f32(Wm, dtype)]
        for r in range(rows):
            for f in range(H * Dh):
                acc = 0.0
                for c in range(d):
                    acc += xf[r][c] * wf[f][c]      # feature f of row r = <W[f,:], x[r,:]>
                assert abs(got[r, f // Dh, f % Dh] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_rotary_is_a_complex_rotation_by_position():
    """Feature pair (i, i + Dh/2) read as the complex number x_i + j x_{i+Dh/2} is multiplied by
    exp(j pos base^(-2i/Dh)): position 0 is the identity, norms are preserved, and the product of a rotated
    query with a rotated key depends on the difference of their positions only."""
    n, H, Dh, base = 6, 3, 16, 10000.0
    x = rng.normal(6, "x", (n, H, Dh)).astype(np.float64)
    pos = np.array([0, 1, 2, 7, 100, 4095])
    y = R.rope_rotate(x, pos, base)
    half = Dh // 2
    for t in range(n):
        for i in range(half):
            w = complex(math.cos(pos[t] * base ** (-2.0 * i / Dh)), math.sin(pos[t] * base ** (-2.0 * i / Dh)))
            for h in range(H):
                z = complex(x[t, h, i], x[t, h, i + half]) * w
                assert abs(y[t, h, i] - z.real) < 1e-9 and abs(y[t, h, i + half] - z.imag) < 1e-9
    assert np.array_equal(y[0], x[0])
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)
    q, k = x[:3], x[3:]
    d0 = np.einsum("thd,thd->th", R.rope_rotate(q, [5, 9, 40], base), R.rope_rotate(k, [2, 9, 31], base))
    d1 = np.einsum("thd,thd->th", R.rope_rotate(q, [105, 1009, 47], base), R.rope_rotate(k, [102, 1009, 38], base))
    assert np.allclose(d0, d1, atol=1e-9)
    # angle of the first pair grows by one radian per position (base^0 = 1), the last pair turns slowest
    e = np.zeros((1, 1, Dh)); e[0, 0, 0] = 1.0
    r = R.rope_rotate(e, [1], base)
    assert abs(r[0, 0, 0] - math.cos(1.0)) < 1e-12 and abs(r[0, 0, half] - math.sin(1.0)) < 1e-12


def test_projecting_kept_rows_equals_compacting_the_full_projection():
    """Row-wise operations commute with the gather of Eq. 5 line 3: projecting (and rotating by ORIGINAL
    positions) only the kept rows gives the kept rows of the full sequence's projection; the cache then holds
    exactly those K/V rows."""
    w = W.make("proj", "bf16", 64, 2, 16, 3, [2, 0, 1], [9, 6, 0], [3, 2, 4], 0.4, 0, project_qkv=True)
    pre, pred, aw = W.prefill_inputs(w), W.predictor(w), W.attn_weights(w)
    vis = np.concatenate([np.arange(w.seq_off[b] + w.n_sys[b], w.seq_off[b] + w.n_sys[b] + w.n_vis[b])
                          for b in range(w.B)]).astype(np.int64)
    D = R.score(pre["hidden"][vis], pred["W1"], pred["b1"], pred["W2"], pred["b2"], w.dtype)
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    total = int(off[-1])
    h_star, _ = R.compact(idx, off, w.seq_off, hidden=pre["hidden"])
    bt, n_pages = W.block_table(w)
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    Q, K, V = R.qkv_project(h_star, off, idx[:total], aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, 10000.0, cache)
    # the other way round: every row of every sequence at its own position, then the gather
    seq_pos = np.concatenate([np.arange(w.seq_off[b + 1] - w.seq_off[b]) for b in range(w.B)])
    Qf, Kf, Vf = R.qkv_project(pre["hidden"], w.seq_off, seq_pos, aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype, 10000.0)
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)])
    assert np.array_equal(Q, Qf[src]) and np.array_equal(K, Kf[src]) and np.array_equal(V, Vf[src])
    # without the rotation the projections are the ones the workload generator made for these hidden states
    Q0, K0, V0 = R.qkv_project(h_star, off, idx[:total], aw["q"], aw["k"], aw["v"], w.H, w.Dh, w.dtype)
    assert np.abs(Q0 - R.widen(pre["Q"], w.dtype)[src]).max() < 0.02 and np.abs(V0 - R.widen(pre["V"], w.dtype)[src]).max() < 0.02
    assert np.array_equal(V0, V)
    for b in range(w.B):
        n = int(off[b + 1] - off[b])
        assert cache.cache_len[b] == n
        Kc, Vc = cache.rows(b)
        assert np.array_equal(Kc, R.narrow(K[off[b]:off[b + 1]], w.dtype))
        assert np.array_equal(Vc, R.narrow(V[off[b]:off[b + 1]], w.dtype))


# ------------------------------------------------------------------ decoding without KV cache (Sec. 3.3.2, Eq. 12)

def test_keep_last_mode_is_the_threshold_rule_with_the_last_entry_set():
    D = rng.normal(11, "D", (40, 2)).astype(np.float32)
    seq_off, v0, n = [0, 12, 12, 40], [2, 0, 5], [7, 0, 20]      # middle sequence empty
    logits = np.concatenate([D[:7], D[7:27]])
    m1, i1, o1 = R.select(logits, seq_off, v0, n, R.THRESHOLD, 0.0, 0.3)
    m2, i2, o2 = R.select(logits, seq_off, v0, n, R.THRESHOLD_KEEP_LAST, 0.0, 0.3)
    want = m1.copy()
    want[0 + 2 + 7 - 1] = 1
    want[12 + 5 + 20 - 1] = 1
    assert np.array_equal(m2, want)
    m3, _, _ = R.select(logits, seq_off, v0, n, R.THRESHOLD_KEEP_LAST, 0.0, float("inf"))
    assert m3[2:9].tolist() == [0] * 6 + [1] and m3[17:37].tolist() == [0] * 19 + [1]   # nothing but the last one


def test_decoding_without_cache_reproduces_decoding_with_cache():
    """Two formulations of the same step.  With KV cache (Eq. 6): the new token attends over the cached kept
    tokens plus itself, and enters the cache only if kept.  Without (Eq. 12 + Eq. 1): all output tokens are
    re-masked with the last one forced to 1, compacted, and attended causally.  The last row of the second must
    equal the output of the first at every step, for any keep history."""
    w = W.make("nocache", "bf16", 64, 2, 16, 2, [1, 0], [6, 4], [2, 3], 0.5, 7, project_qkv=True)
    pre, dec = W.prefill_inputs(w), W.decode_inputs(w)
    D = rng.normal(w.seed, "D", (int(sum(w.n_vis)), 2)).astype(np.float32)
    mask, idx, off = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, w.keep_ratio, 0.0)
    bt, n_pages = W.block_table(w)
    cache = R.PagedCache(n_pages, bt, w.H, w.Dh, w.dtype)
    _, Qp = R.compact(idx, off, w.seq_off, Q=pre["Q"], K=pre["K"], V=pre["V"], cache=cache)
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)])
    Kp, Vp = pre["K"][src], pre["V"][src]
    scale = 1.0 / math.sqrt(w.Dh)
    logits = rng.normal(w.seed, "ot.logits", (w.T, w.B, 2)).astype(np.float32)   # predictor logits of the output tokens
    for t in range(w.T):
        keep = R.decode_keep(logits[t], 0.0)
        o_cache, err = R.decode_attn_append(dec["q"][t], dec["k"][t], dec["v"][t], keep, cache, scale)
        assert not err.any()
        # without cache: all output tokens 0..t of both sequences, sequence-major
        n_ot = t + 1
        seqmaj = lambda a: np.concatenate([a[:n_ot, b] for b in range(w.B)])
        o_off = np.arange(w.B + 1) * n_ot
        O, ooff, m = R.decode_nocache_step(Qp, Kp, Vp, off, seqmaj(dec["q"]), seqmaj(dec["k"]), seqmaj(dec["v"]),
                                           o_off, seqmaj(logits), 0.0, scale, w.dtype)
        for b in range(w.B):
            assert np.allclose(O[ooff[b + 1] - 1], o_cache[b], rtol=0, atol=1e-12)
            # kept output tokens = the history of keep decisions, plus the current token
            hist = [int(R.decode_keep(logits[s], 0.0)[b]) for s in range(t)] + [1]
            n_p = int(off[b + 1] - off[b])
            assert ooff[b + 1] - ooff[b] == n_p + sum(hist)
            assert int(cache.cache_len[b]) == n_p + sum(hist[:-1]) + int(keep[b])
