"""Pins of the paper-form predictor oracle (Appendix A.4.1) against things other than itself: library routines
in float64, brute-force loops, and the invariances the architecture has."""
import math

import numpy as np
import pytest
import torch

from oracle import dllava_ref as R
from oracle import predictor_ref as PR
from synth import workloads as W


def _wl(dtype="f32", d=64, seed=11):
    return W.make("pp", dtype, d, 2, 64, 2, [0, 0], [5, 3], [0, 0], 0.5, 1, seed=seed)


def _x(w, M, tag="x"):
    from synth import rng
    return W.store(rng.normal(w.seed, tag, (M, w.d)), w.dtype)


def test_layer_norm_matches_library_routine():
    r = np.random.RandomState(0)
    z, g, b = r.randn(7, 512) * 3 + 1, r.rand(512) + 0.5, r.randn(512)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(z), (512,), torch.from_numpy(g), torch.from_numpy(b), PR.LN_EPS)
    assert np.abs(PR.layer_norm(z, g, b) - ref.numpy()).max() < 1e-12
    y = PR.layer_norm(z, np.ones(512), np.zeros(512))
    assert np.abs(y.mean(axis=1)).max() < 1e-12 and np.abs(y.var(axis=1) - 1).max() < 1e-5


def test_attention_matches_loops_and_library():
    r = np.random.RandomState(1)
    n = 6
    q, k, v = r.randn(n, 512), r.randn(n, 512), r.randn(n, 512)
    out = PR.attention(q, k, v)
    # pure loops, head by head, query by query
    for h in (0, 3, 7):
        for i in range(n):
            s = [sum(q[i, h * 64 + c] * k[j, h * 64 + c] for c in range(64)) / 8.0 for j in range(n)]
            m = max(s)
            p = [math.exp(t - m) for t in s]
            for c in (0, 17, 63):
                o = sum(p[j] * v[j, h * 64 + c] for j in range(n)) / sum(p)
                assert abs(out[i, h * 64 + c] - o) < 1e-12
    t = lambda a: torch.from_numpy(a).reshape(n, 8, 64).transpose(0, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v)).transpose(0, 1).reshape(n, 512)
    assert np.abs(out - ref.numpy()).max() < 1e-12


def _torch_block(blk):
    """The library's pre-norm encoder layer carrying the same weights (float64)."""
    f = lambda a: torch.from_numpy(R.widen(a, "f32") if a.dtype != np.float32 or a.ndim == 2 else a.astype(np.float64))
    layer = torch.nn.TransformerEncoderLayer(512, 8, 2048, dropout=0.0, activation="gelu", layer_norm_eps=PR.LN_EPS,
                                             batch_first=True, norm_first=True, dtype=torch.float64)
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(f(blk["Wqkv"])); layer.self_attn.in_proj_bias.copy_(f(blk["bqkv"]))
        layer.self_attn.out_proj.weight.copy_(f(blk["Wo"])); layer.self_attn.out_proj.bias.copy_(f(blk["bo"]))
        layer.linear1.weight.copy_(f(blk["Wfc1"])); layer.linear1.bias.copy_(f(blk["bfc1"]))
        layer.linear2.weight.copy_(f(blk["Wfc2"])); layer.linear2.bias.copy_(f(blk["bfc2"]))
        layer.norm1.weight.copy_(f(blk["ln1_g"])); layer.norm1.bias.copy_(f(blk["ln1_b"]))
        layer.norm2.weight.copy_(f(blk["ln2_g"])); layer.norm2.bias.copy_(f(blk["ln2_b"]))
    return layer.eval()


def test_block_matches_library_encoder_layer():
    """A dropped residual, a wrong norm placement, a transposed weight or a mis-cut q|k|v would all show here."""
    w = _wl()
    P = W.paper_predictor(w, 2)
    r = np.random.RandomState(2)
    z = r.randn(8, 512)
    off = np.array([0, 5, 8])
    for blk in P["blocks"]:
        got = PR.vit_block(z, off, blk, "f32", rnd=False)
        layer = _torch_block(blk)
        with torch.no_grad():
            ref = np.concatenate([layer(torch.from_numpy(z[a:b])[None])[0].numpy() for a, b in ((0, 5), (5, 8))])
        assert np.abs(got - ref).max() < 1e-10


def test_text_predictor_matches_plain_loops():
    w = _wl(d=16)
    P = W.paper_predictor(w, 0)
    x = _x(w, 2)
    got = PR.predict(x, None, P, "f32", round_intermediates=False)
    g = lambda t: 0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0)))
    for m in range(2):
        z = [sum(float(x[m, c]) * float(P["W_in"][u, c]) for c in range(16)) + float(P["b_in"][u]) for u in range(512)]
        h1 = [g(sum(z[c] * float(P["W_h1"][u, c]) for c in range(512)) + float(P["b_h1"][u])) for u in range(256)]
        h2 = [g(sum(h1[c] * float(P["W_h2"][u, c]) for c in range(256)) + float(P["b_h2"][u])) for u in range(128)]
        for o in range(2):
            D = sum(h2[c] * float(P["W_h3"][o, c]) for c in range(128)) + float(P["b_h3"][o])
            assert abs(float(got[m, o]) - D) < 1e-6   # float32 output


def test_image_predictor_is_the_composition_and_mixes_only_within_a_span():
    w = _wl()
    P = W.paper_predictor(w, 2)
    x = _x(w, 8)
    off = np.array([0, 5, 8])
    D = PR.predict(x, off, P, "f32", round_intermediates=False)
    # composition written out with the library layers
    z = PR.linear(R.widen(x, "f32"), P["W_in"], P["b_in"], "f32")
    with torch.no_grad():
        for blk in P["blocks"]:
            layer = _torch_block(blk)
            z = np.concatenate([layer(torch.from_numpy(z[a:b])[None])[0].numpy() for a, b in ((0, 5), (5, 8))])
    h = R.gelu(PR.linear(R.gelu(PR.linear(z, P["W_h1"], P["b_h1"], "f32")), P["W_h2"], P["b_h2"], "f32"))
    assert np.abs(D - PR.linear(h, P["W_h3"], P["b_h3"], "f32")).max() < 1e-6
    # tokens of another sequence do not matter
    x2 = x.copy()
    x2[5:] = _x(w, 3, "other")
    D2 = PR.predict(x2, off, P, "f32", round_intermediates=False)
    assert np.array_equal(D[:5], D2[:5]) and not np.allclose(D[5:], D2[5:])
    # no position term: permuting a span's tokens permutes its logits
    perm = np.array([3, 0, 4, 1, 2])
    x3 = x.copy()
    x3[:5] = x[:5][perm]
    D3 = PR.predict(x3, off, P, "f32", round_intermediates=False)
    assert np.abs(D3[:5] - D[:5][perm]).max() < 1e-5
    # the mixing is real: changing one token of a span changes the others' logits
    x4 = x.copy()
    x4[0] = _x(w, 1, "swap")[0]
    D4 = PR.predict(x4, off, P, "f32", round_intermediates=False)
    assert np.abs(D4[1:5] - D[1:5]).max() > 1e-4


def test_text_predictor_rows_are_independent_and_blocks_change_the_result():
    w = _wl("bf16")
    P0, P2 = W.paper_predictor(w, 0), W.paper_predictor(w, 2)
    x = _x(w, 8)
    D = PR.predict(x, None, P0, "bf16")
    for m in (0, 3, 7):
        assert np.array_equal(PR.predict(x[m:m + 1], None, P0, "bf16"), D[m:m + 1])
    assert D.dtype == np.float32 and D.shape == (8, 2)
    assert not np.allclose(PR.predict(x, np.array([0, 5, 8]), P2, "bf16"), D, atol=1e-3)


def test_stored_intermediates_cost_little():
    """Rounding every stored tensor to bfloat16 (8 significant bits, a dozen tensors deep) moves logits of order 1 by
    about 1e-2: the roundings are part of what is computed, which is why the oracle applies them."""
    w = _wl("bf16", d=256)
    P = W.paper_predictor(w, 2)
    x = _x(w, 40)
    off = np.array([0, 25, 40])
    a = PR.predict(x, off, P, "bf16", round_intermediates=True)
    b = PR.predict(x, off, P, "bf16", round_intermediates=False)
    assert 1e-4 < np.abs(a - b).max() < 5e-2


def test_flop_count_formula():
    # one block, one span of n tokens: 2*M*(12*512^2) for the linear layers and 4*n^2*512 for the two products
    n, d = 10, 64
    head = 2.0 * n * (d * 512 + 512 * 256 + 256 * 128 + 256)
    assert PR.predict_flops(n, d, [n], 0) == head
    assert PR.predict_flops(n, d, [n], 1) - head == 2.0 * n * 12 * 512 * 512 + 4.0 * n * n * 512
