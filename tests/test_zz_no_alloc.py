"""dllava_decode_attn_append_static (the decode step for callers that cannot bring a workspace: its counters and partial
results live in a device array inside the library) against dllava_decode_attn_append on the same inputs: two calls in
a row on the shared array, the second with a smaller input, then a shape without split launches; outputs, decisions,
lengths and every page must be identical bit for bit (same kernels, same launch shapes)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2412_00876_amd as P
from synth import rng
from synth import workloads as W


def _H():
    from tests import harness
    return harness


def _state(h, tag, B, H, Dh, max_len, T):
    """Two identical caches with seeded ragged lengths, and T steps of decode inputs."""
    w = W.make(tag, "bf16", 256, H, Dh, B, 0, 0, 0, 1.0, T)
    rs = np.random.RandomState(B * 1000 + H)
    lens = rs.randint(0, max_len, size=B).astype(np.int32)
    lens[0] = 0
    mp = (int(lens.max()) + T) // 16 + 2
    bt = rng.permutation(11, f"bt{tag}", B * mp).reshape(B, mp).astype(np.int32)
    pages_np = W.store(rng.normal(11, f"pages{tag}", (B * mp, 2, H, 16, Dh)), "bf16")
    paths = []
    for _ in range(2):
        g = h.GpuPath(w, None, None, n_pages=B * mp, bt=bt)
        g.pages.copy_(h.to_dev(pages_np, "bf16"))
        g.cache_len.copy_(torch.from_numpy(lens))
        paths.append(g)
    return w, paths, W.decode_inputs(w, T)


def _steps(h, tag, B, H, Dh, max_len, T=3):
    w, (g_ws, g_st), dec = _state(h, tag, B, H, Dh, max_len, T)
    for t in range(T):
        keep = torch.from_numpy(rng.bernoulli(11, f"keep{tag}{t}", (B,), 0.5)).to(h.DEV)
        q, k, v = (h.to_dev(dec[n][t], "bf16") for n in ("q", "k", "v"))
        print(f"no-alloc decode: {tag} B={B} H={H} Dh={Dh} step {t}", flush=True)
        o_ws, keep_ws = g_ws.decode(q, k, v, keep_override=keep)
        o_st = torch.zeros_like(q)
        keep_st = torch.full((B,), 255, dtype=torch.uint8, device=h.DEV)
        P.dllava_decode_attn_append_static(q, k, v, B, None, 0.0, keep, g_st.cache, g_st.scale, o_st, keep_st, g_st.err)
        torch.cuda.synchronize()
        assert torch.equal(o_st.view(torch.int16), o_ws.view(torch.int16)), f"{tag} step {t}: o"
        assert torch.equal(keep_st, keep_ws), f"{tag} step {t}: keep"
        assert torch.equal(g_st.cache_len, g_ws.cache_len), f"{tag} step {t}: cache_len"
    assert torch.equal(g_st.pages.view(torch.int16), g_ws.pages.view(torch.int16)), f"{tag}: pages"
    assert int(g_st.err.item()) == 0 and int(g_ws.err.item()) == 0


def test_static_scratch_decode_matches_the_workspace_form():
    h = _H()
    _steps(h, "large", 6, 8, 128, 300)      # several blocks per (sequence, head): counters and partial results in use
    _steps(h, "small", 2, 3, 128, 40)       # a smaller input right after, on the same array
    _steps(h, "wide", 20, 32, 128, 120)     # one block per (sequence, head): counters only
    _steps(h, "dh64", 3, 5, 64, 90)


def test_static_scratch_decode_refuses_what_does_not_fit():
    h = _H()
    B, H = 400, 16   # 2*B*H + B = 13200 counters > 12288
    w = W.make("toolarge", "bf16", 256, H, 64, B, 0, 0, 0, 1.0, 1)
    bt = np.arange(B, dtype=np.int32).reshape(B, 1)
    g = h.GpuPath(w, None, None, n_pages=B, bt=bt)
    q = torch.zeros((B, H, 64), dtype=torch.bfloat16, device=h.DEV)
    keep = torch.zeros(B, dtype=torch.uint8, device=h.DEV)
    with pytest.raises(P.DllavaError) as e:
        P.dllava_decode_attn_append_static(q, q, q, B, None, 0.0, keep, g.cache, g.scale, torch.zeros_like(q), None, g.err)
    assert e.value.status == -5 and "workspace" in str(e.value)
