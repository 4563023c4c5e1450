"""GPU parity of dllava_masked_attn (attention of the training form, Eq. 7: the keep mask inside the softmax on the
full token set) against the oracle: ragged batches with random masks, the all-ones and all-zeros masks, long runs of
dropped tokens, the identity with attention over the compacted sequence, and sequences longer than the kernel's
in-register mask words."""
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


def _qkv(seed, rows, H, Dh):
    return tuple(W.store(rng.normal(seed, t, (rows, H, Dh)), "bf16") for t in "qkv")


def _assert_one_step(a, b, what):
    """Two bfloat16 results of the same quantity: at most one rounding step apart."""
    assert (np.abs(a - b) <= 2.0 ** -7 * np.abs(b) + 2e-3).all(), (what, float(np.abs(a - b).max()))


def _run(h, q, k, v, off, keep, H, Dh):
    rows, B = q.shape[0], len(off) - 1
    O = torch.full((rows, H, Dh), float("nan"), dtype=torch.bfloat16, device=h.DEV)
    ws = torch.full((P.dllava_masked_attn_workspace(rows, B),), 0x5a, dtype=torch.uint8, device=h.DEV)
    P.dllava_masked_attn(h.to_dev(q, "bf16"), h.to_dev(k, "bf16"), h.to_dev(v, "bf16"), B,
                         torch.from_numpy(np.asarray(off, np.int32)).to(h.DEV), rows, H, Dh, 1.0 / math.sqrt(Dh),
                         torch.from_numpy(np.asarray(keep, np.uint8)).to(h.DEV), O, P.BF16, ws)
    return O


@pytest.mark.parametrize("lens,H,Dh,p", [([130, 1, 300], 4, 128, 0.5), ([33, 0, 64, 97], 3, 64, 0.3),
                                          ([257], 2, 128, 0.9), ([5, 700], 2, 64, 0.1)])
def test_masked_attention_matches_oracle(lens, H, Dh, p):
    h = _H()
    rows = int(sum(lens))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v = _qkv(40 + H + Dh, rows, H, Dh)
    keep = rng.bernoulli(41, "keep", (rows,), p).astype(np.uint8) * 3      # any non-zero value means kept
    O = _run(h, q, k, v, off, keep, H, Dh)
    ref = R.masked_attn(q, k, v, off, keep, 1.0 / math.sqrt(Dh), "bf16")
    _assert_out_close(h.as_f64(O), ref, "bf16", "masked attention")


def test_masked_attention_special_masks_and_the_compacted_form():
    h = _H()
    lens, H, Dh = [200, 90], 4, 128
    rows = sum(lens)
    off = np.array([0, 200, 290], np.int32)
    q, k, v = _qkv(50, rows, H, Dh)
    scale = 1.0 / math.sqrt(Dh)
    dev = lambda a: h.to_dev(a, "bf16")
    # nothing kept: every row sees itself only and returns its own value, exactly
    O0 = _run(h, q, k, v, off, np.zeros(rows, np.uint8), H, Dh)
    assert np.array_equal(h.bits(O0), v)
    # everything kept: causal attention
    O1 = _run(h, q, k, v, off, np.ones(rows, np.uint8), H, Dh)
    Oc = torch.zeros_like(O1)
    P.dllava_prefill_attn(dev(q), dev(k), dev(v), None, 2, torch.from_numpy(off).to(h.DEV), rows, H, Dh, scale, Oc, P.BF16)
    _assert_one_step(h.as_f64(O1), h.as_f64(Oc), "all kept against causal attention")
    assert (O1 != Oc).float().mean().item() <= 0.01
    # a long run of dropped tokens at the start and in the middle (whole key tiles without a visible key)
    keep = np.ones(rows, np.uint8)
    keep[0:101] = 0
    keep[130:199] = 0
    keep[200:290] = 0
    keep[289] = 1
    O2 = _run(h, q, k, v, off, keep, H, Dh)
    ref = R.masked_attn(q, k, v, off, keep, scale, "bf16")
    _assert_out_close(h.as_f64(O2), ref, "bf16", "runs of dropped tokens")
    # on the kept rows: attention over the compacted sequences (the inference form of the same thing)
    idx = np.flatnonzero(keep)
    off_c = np.array([0, int(keep[:200].sum()), int(keep.sum())], np.int32)
    Ok = torch.zeros((len(idx), H, Dh), dtype=torch.bfloat16, device=h.DEV)
    P.dllava_prefill_attn(dev(q[idx]), dev(k[idx]), dev(v[idx]), None, 2, torch.from_numpy(off_c).to(h.DEV), len(idx), H, Dh,
                          scale, Ok, P.BF16)
    _assert_one_step(h.as_f64(O2)[idx], h.as_f64(Ok), "kept rows against the compacted form")


@pytest.mark.parametrize("n", [2500, 8300])
def test_masked_attention_long_sequences(n):
    """More key tiles than one register of mask words holds (64), and more than the four registers hold (256)."""
    h = _H()
    H, Dh = 1, 64
    lens = [70, n]
    rows = sum(lens)
    off = np.array([0, 70, 70 + n], np.int32)
    q, k, v = _qkv(60 + n, rows, H, Dh)
    keep = rng.bernoulli(61, "keep", (rows,), 0.4).astype(np.uint8)
    O = _run(h, q, k, v, off, keep, H, Dh)
    some = sorted({0, 69, 70, 71, 70 + 2047, 70 + 2048, 70 + 2049, rows - 1, rows - 2, 70 + n // 2} |
                  set(int(x) for x in rng.permutation(62, "rows", rows)[:24]))
    ref = R.masked_attn_rows(q, k, v, off, keep, 1.0 / math.sqrt(Dh), "bf16", some)
    _assert_out_close(h.as_f64(O)[some], ref, "bf16", "sampled rows of a long sequence")
    assert torch.isfinite(O.float()).all()


def test_many_sequences_take_the_other_block_numbering():
    """More than 64 sequences: the kernel numbers its blocks sequence by sequence instead of with ballots; both the
    masked (Eq. 7) and the unmasked-span forms go through it."""
    from oracle import predictor_ref as PR
    h = _H()
    B, H, Dh = 70, 2, 64
    lens = [int(x) for x in (rng.uniform01(70, "lens", 0, B) * 60).astype(int)]     # 0..59 rows each, some empty
    lens[3] = 0
    lens[10] = 200
    rows = int(sum(lens))
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v = _qkv(71, rows, H, Dh)
    keep = rng.bernoulli(72, "keep", (rows,), 0.5).astype(np.uint8)
    O = _run(h, q, k, v, off, keep, H, Dh)
    _assert_out_close(h.as_f64(O), R.masked_attn(q, k, v, off, keep, 1.0 / math.sqrt(Dh), "bf16"), "bf16", "70 sequences")
    # unmasked attention within each span (the image predictor's token mixing)
    Os = torch.zeros((rows, H, Dh), dtype=torch.bfloat16, device=h.DEV)
    P.dllava_span_attn(h.to_dev(q, "bf16"), h.to_dev(k, "bf16"), h.to_dev(v, "bf16"), B, torch.from_numpy(off).to(h.DEV),
                       rows, H, Dh, 1.0 / math.sqrt(Dh), Os, P.BF16)
    ref = np.zeros((rows, H * Dh))
    f = lambda a: R.widen(a, "bf16").reshape(len(a), H * Dh)
    for a, b in zip(off[:-1], off[1:]):
        if b > a:
            ref[a:b] = PR.attention(f(q[a:b]), f(k[a:b]), f(v[a:b]), heads=H)
    _assert_out_close(h.as_f64(Os).reshape(rows, H * Dh), ref, "bf16", "70 spans")
