"""Pins of the decoder-stack oracle against things other than itself: the reference implementation of the LLaMA decoder
layer in the `transformers` package (float64, same weights), library RMSNorm / SiLU, and the structure of the one-time
reduction (layers up to l see every token, later layers the kept ones at their original positions)."""
import math

import numpy as np
import pytest
import torch

from oracle import decoder_ref as DR
from oracle import dllava_ref as R
from synth import rng
from synth import workloads as W


def _wl(dtype="f32", seed=5):
    return W.make("dec", dtype, 64, 2, 32, 2, [2, 1], [9, 6], [3, 4], 0.5, 1, seed=seed)


def test_rms_norm_and_silu_match_library_routines():
    r = np.random.RandomState(0)
    x, g = r.randn(5, 64) * 2, r.rand(64) + 0.5
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), DR.RMS_EPS)
    assert np.abs(DR.rms_norm(x, g) - ref.numpy()).max() < 1e-12
    assert np.abs(DR.silu(x) - torch.nn.functional.silu(torch.from_numpy(x)).numpy()).max() < 1e-12


def _hf_layer(Lw, d, dff, H, Dh):
    from transformers import LlamaConfig
    from transformers.models.llama.modeling_llama import LlamaDecoderLayer, LlamaRotaryEmbedding
    cfg = LlamaConfig(hidden_size=d, intermediate_size=dff, num_attention_heads=H, num_key_value_heads=H, head_dim=Dh,
                      rms_norm_eps=DR.RMS_EPS, rope_theta=DR.ROPE_BASE, attention_bias=False, mlp_bias=False,
                      attn_implementation="eager")
    layer = LlamaDecoderLayer(cfg, 0).double().eval()
    f = lambda a: torch.from_numpy(np.asarray(a, np.float32).astype(np.float64))
    with torch.no_grad():
        layer.self_attn.q_proj.weight.copy_(f(Lw["Wq"])); layer.self_attn.k_proj.weight.copy_(f(Lw["Wk"]))
        layer.self_attn.v_proj.weight.copy_(f(Lw["Wv"])); layer.self_attn.o_proj.weight.copy_(f(Lw["Wo"]))
        layer.mlp.gate_proj.weight.copy_(f(Lw["Wg"])); layer.mlp.up_proj.weight.copy_(f(Lw["Wu"]))
        layer.mlp.down_proj.weight.copy_(f(Lw["Wd"]))
        layer.input_layernorm.weight.copy_(f(Lw["g1"])); layer.post_attention_layernorm.weight.copy_(f(Lw["g2"]))
    return layer, LlamaRotaryEmbedding(cfg)


def test_layer_matches_the_reference_llama_layer():
    """A wrong rotary pairing, a missing residual, a transposed projection or a swapped gate/up would all show here;
    the positions are NOT 0..n-1 (kept tokens keep their original positions)."""
    w = _wl()
    Lw = W.decoder_layers(w, 1, 96)[0]
    n = 7
    x = rng.normal(3, "x", (n, w.d)).astype(np.float64)
    pos = np.array([0, 1, 4, 5, 9, 20, 21])
    got = DR.decoder_layer(x, np.array([0, n]), pos, Lw, w.H, w.Dh, "f32", round_intermediates=False)
    layer, rot = _hf_layer(Lw, w.d, 96, w.H, w.Dh)
    xt, pt = torch.from_numpy(x)[None], torch.from_numpy(pos)[None]
    cos, sin = rot(xt, pt)
    mask = torch.full((n, n), float("-inf"), dtype=torch.float64).triu(1)[None, None]
    with torch.no_grad():
        ref = layer(xt, attention_mask=mask, position_ids=pt, position_embeddings=(cos.double(), sin.double()))
    ref = (ref[0] if isinstance(ref, tuple) else ref)[0].numpy()
    assert np.abs(got - ref).max() < 2e-5          # the library takes cos / sin in float32


def test_stack_reduces_once_and_keeps_original_positions():
    w = _wl()
    layers = W.decoder_layers(w, 3, 96)
    pred = W.predictor(w)
    x0 = W.store(rng.normal(w.seed, "h0", (w.sumN, w.d)), "f32")
    predictor = lambda rows: R.score(rows, pred["W1"], pred["b1"], pred["W2"], pred["b2"], "f32")
    xf, idx, off, logits = DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, 1, 0.5, predictor, w.H, w.Dh,
                                              "f32", round_intermediates=False)
    # by hand: layer 0 on everything, decision, layers 1-2 on the kept rows with their original positions
    pos_all = np.concatenate([np.arange(n) for n in np.diff(w.seq_off)])
    x1 = DR.decoder_layer(R.widen(x0, "f32"), w.seq_off, pos_all, layers[0], w.H, w.Dh, "f32", False)
    vis = np.concatenate([np.arange(w.seq_off[b] + w.vis_start[b], w.seq_off[b] + w.vis_start[b] + w.vis_len[b])
                          for b in range(w.B)])
    D = predictor(R.narrow(x1[vis], "f32"))
    mask, idx2, off2 = R.select(D, w.seq_off, w.vis_start, w.vis_len, R.TOPK, 0.5, 0.0)
    assert np.array_equal(idx, idx2) and np.array_equal(off, off2) and np.array_equal(logits, D)
    assert int(off[-1]) == int(mask.sum()) < w.sumN
    src = np.concatenate([w.seq_off[b] + idx[off[b]:off[b + 1]] for b in range(w.B)])
    x = x1[src]
    for L in layers[1:]:
        x = DR.decoder_layer(x, off, idx[:off[-1]], L, w.H, w.Dh, "f32", False)
    assert np.array_equal(xf, x)
    # l beyond the stack: nothing is reduced; l = 0: reduced before the first layer
    xa, ia, oa, _ = DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, 3, 0.5, predictor, w.H, w.Dh, "f32", False)
    assert xa.shape[0] == w.sumN and np.array_equal(oa, w.seq_off)
    xb, ib, ob, _ = DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, 0, 0.5, predictor, w.H, w.Dh, "f32", False)
    assert xb.shape[0] == int(ob[-1]) < w.sumN


def test_layer_attention_equals_the_path_oracle():
    """The layer's attention part is dllava_ref's projection + causal attention: same numbers through either."""
    w = _wl("bf16")
    Lw = W.decoder_layers(w, 1, 96)[0]
    n = w.sumN
    x = W.store(rng.normal(9, "x", (n, w.d)), "bf16")
    pos = np.concatenate([np.arange(k) for k in np.diff(w.seq_off)])
    h1 = R.narrow(DR.rms_norm(R.widen(x, "bf16"), Lw["g1"]), "bf16")
    Q, K, V = R.qkv_project(h1, w.seq_off, pos, Lw["Wq"], Lw["Wk"], Lw["Wv"], w.H, w.Dh, "bf16", DR.ROPE_BASE)
    A = R.prefill_attn(R.narrow(Q, "bf16"), R.narrow(K, "bf16"), R.narrow(V, "bf16"), w.seq_off, 1 / math.sqrt(w.Dh), "bf16")
    xa = R.widen(x, "bf16") + R.widen(R.narrow(A.reshape(n, -1), "bf16"), "bf16") @ R.widen(Lw["Wo"], "bf16").T
    # replay the layer with the feed-forward weights zeroed: what is left is the attention half
    L0 = dict(Lw, Wd=np.zeros_like(Lw["Wd"]))
    got = DR.decoder_layer(R.widen(x, "bf16"), w.seq_off, pos, L0, w.H, w.Dh, "bf16", True)
    assert np.array_equal(got, R.widen(R.narrow(xa, "bf16"), "bf16"))


def test_decode_step_equals_prefill_of_the_extended_sequence():
    """With every generated token kept, a decode step through the stack (caches) gives the last row of a prefill over
    the sequence extended by that token; with tokens dropped, later layers' caches stay shorter while layers before l
    keep everything (Sec. 3.3: the decision is taken once and shared by the subsequent layers)."""
    w = _wl()
    n_layers, l, T = 3, 1, 3
    layers = W.decoder_layers(w, n_layers, 96)
    B, d = w.B, w.d
    n0 = np.diff(w.seq_off)
    x0 = W.store(rng.normal(w.seed, "h0", (w.sumN, d)), "f32")
    xs = [W.store(rng.normal(w.seed, f"new{t}", (B, d)), "f32") for t in range(T)]
    no_pred = lambda rows: np.tile(np.array([[0.0, 1.0]], np.float32), (len(rows), 1))      # margin +1: keep
    mk = lambda: [R.PagedCache(B * 4, np.arange(B * 4, dtype=np.int32).reshape(B, 4), w.H, w.Dh, "f32") for _ in layers]
    caches = mk()
    DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, n_layers, 1.0, no_pred, w.H, w.Dh, "f32", False, caches)
    outs = []
    for t in range(T):
        xo, keep, _ = DR.decoder_decode_step(xs[t], n0 + t, layers, caches, l, 0.0, no_pred, w.H, w.Dh, "f32", False)
        assert keep.all()
        outs.append(xo)
    # the same through one prefill over the extended sequences
    ext = np.concatenate([np.concatenate([x0[w.seq_off[b]:w.seq_off[b + 1]]] + [xs[t][b:b + 1] for t in range(T)])
                          for b in range(B)])
    off_e = np.concatenate([[0], np.cumsum(n0 + T)])
    xe, _, _, _ = DR.decoder_prefill(ext, off_e, w.vis_start, w.vis_len, layers, n_layers, 1.0, no_pred, w.H, w.Dh, "f32", False)
    for t in range(T):
        for b in range(B):
            assert np.abs(outs[t][b] - xe[off_e[b] + n0[b] + t]).max() < 1e-4      # K/V pass through float32 storage
    # dropped tokens: layers >= l do not grow, layers < l do
    caches = mk()
    DR.decoder_prefill(x0, w.seq_off, w.vis_start, w.vis_len, layers, n_layers, 1.0, no_pred, w.H, w.Dh, "f32", False, caches)
    drop = lambda rows: np.tile(np.array([[1.0, 0.0]], np.float32), (len(rows), 1))
    for t in range(T):
        _, keep, _ = DR.decoder_decode_step(xs[t], n0 + t, layers, caches, l, 0.0, drop, w.H, w.Dh, "f32", False)
        assert not keep.any()
    assert list(caches[0].cache_len) == list(n0 + T) and list(caches[1].cache_len) == list(n0) == list(caches[2].cache_len)
