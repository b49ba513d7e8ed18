"""Pins for oracle.lm.DecoderLM and its sessions.

The decoder is checked against an independently written PyTorch CPU model built from
library routines (F.rms_norm, complex-number rotary, F.scaled_dot_product_attention,
F.silu), against invariants (causality, shift invariance of rotary attention) and
against the closed form for the logit spread; the cached / tree-masked session is
checked against the from-scratch definition."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle.lm import CachedSession, DecoderLM, RecomputeSession, round_bf16

TINY = si.ModelShape(2, 32, 4, 2, 8, 48, 50, "fp32")
TINY_BF16 = si.ModelShape(2, 32, 4, 2, 8, 48, 50, "bf16")


def _lm(shape, seed=5):
    return DecoderLM(shape, si.make_weights(shape, seed, "target", threads=1))


def _torch_reference(shape, weights, tokens, pos0=0):
    """fp64 decoder from torch library ops; rotary as complex multiplication."""
    W = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in weights.items()}
    H, KVH, hd, f = shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn
    T = len(tokens)
    h = F.embedding(torch.tensor(tokens), W["embed"])
    freqs = shape.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = (torch.arange(T, dtype=torch.float64) + pos0)[:, None] * freqs[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                       # e^{i pos w}

    def rope(x):                                                        # x [T, heads, hd], pairs (i, i+hd/2)
        z = torch.complex(x[..., :hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape.n_layers):
        a = F.rms_norm(h, (shape.d_model,), W[f"L{l}.g_attn"], shape.rms_eps)
        q, k, v = F.linear(a, W[f"L{l}.w_qkv"]).split([H * hd, KVH * hd, KVH * hd], dim=-1)
        q, k, v = rope(q.view(T, H, hd)), rope(k.view(T, KVH, hd)), v.view(T, KVH, hd)
        k = k.repeat_interleave(H // KVH, dim=1)
        v = v.repeat_interleave(H // KVH, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(T, H * hd), W[f"L{l}.w_o"])
        u = F.rms_norm(h, (shape.d_model,), W[f"L{l}.g_ffn"], shape.rms_eps)
        gate, up = F.linear(u, W[f"L{l}.w_gu"]).split([f, f], dim=-1)
        h = h + F.linear(F.silu(gate) * up, W[f"L{l}.w_d"])
    return F.linear(F.rms_norm(h, (shape.d_model,), W["g_final"], shape.rms_eps), W["unembed"]).numpy()


def test_decoder_matches_torch_library_model():
    w = si.make_weights(TINY, 5, "target", threads=1)
    w = {k: (v * 8 if v.ndim == 2 and k != "unembed" else v) for k, v in w.items()}   # make attention non-trivial
    toks = list(np.random.default_rng(0).integers(0, TINY.vocab, 11))
    got = DecoderLM(TINY, w).logits_full(toks)
    want = _torch_reference(TINY, w, toks)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-10)


def test_causality_and_rotary_shift_invariance():
    lm = _lm(TINY)
    toks = list(np.random.default_rng(1).integers(0, TINY.vocab, 9))
    full = lm.logits_full(toks)
    other = toks[:5] + [(t + 1) % TINY.vocab for t in toks[5:]]
    assert np.allclose(lm.logits_full(other)[:5], full[:5], atol=1e-12)
    # rotary attention depends on position differences only
    pk, pv = lm.empty_cache()
    vis = np.tril(np.ones((9, 9), bool))
    shifted = lm.forward_rows(toks, np.arange(9) + 37, pk, pv, vis)[0]
    assert np.allclose(shifted, full, atol=1e-9)


def test_logit_spread_closed_form():
    # unembedding rows ~ N(0, 9/d), final hidden state has unit RMS => logit std = 3
    shape = si.ModelShape(1, 256, 4, 4, 64, 688, 1024, "fp32")
    lm = _lm(shape)
    logits = lm.logits_full(list(range(16)))
    assert abs(logits.std() - 3.0) < 0.15


@pytest.mark.parametrize("shape", [TINY, TINY_BF16], ids=["fp32", "bf16"])
def test_cached_tree_session_equals_full_recompute(shape):
    lm = _lm(shape, seed=9)
    lm.W = {k: (v * 6 if v.ndim == 2 and k != "unembed" else v) for k, v in lm.W.items()}
    if shape.dtype == "bf16":
        lm.W = {k: round_bf16(v) for k, v in lm.W.items()}
    ctx = list(np.random.default_rng(2).integers(0, shape.vocab, 7))
    ref, fast = RecomputeSession(lm, ctx), CachedSession(lm, ctx)
    # bf16 mode rounds at the same points in both forms, so both stay equal to summation order
    tol = dict(rtol=1e-9, atol=1e-9)
    # call 1: root only; call 2: three siblings; call 3: children, one hanging off a node of the same call
    for parents, toks in ([], []), ([-1, -1, -1], [3, 4, 5]), ([0, 2, 4], [6, 7, 8]):
        a, ia = ref.tree_logits(parents, toks)
        b, ib = fast.tree_logits(parents, toks)
        assert ia == ib and np.allclose(a, b, **tol)
    # commit the branch root -> node 2 -> node 4 -> node 5 plus an extra token, then go on
    ref.commit(5, [11]); fast.commit(5, [11])
    assert ref.context == fast.context == ctx + [5, 7, 8, 11]
    a, _ = ref.tree_logits([-1, 0], [1, 2])
    b, _ = fast.tree_logits([-1, 0], [1, 2])
    assert np.allclose(a, b, **tol)
    # two pending context tokens at once (what the draft sees after a fully accepted draft)
    ref.commit(None, [20, 21]); fast.commit(None, [20, 21])
    a, _ = ref.tree_logits([-1], [9]); b, _ = fast.tree_logits([-1], [9])
    assert np.allclose(a, b, **tol)


def test_sibling_order_does_not_change_node_outputs():
    lm = _lm(TINY, seed=3)
    ctx = [1, 2, 3, 4]
    s1, s2 = CachedSession(lm, ctx), CachedSession(lm, ctx)
    a, _ = s1.tree_logits([-1, -1, 0, 1], [10, 11, 12, 13])
    b, _ = s2.tree_logits([-1, -1, 0, 1], [11, 10, 13, 12])
    assert np.allclose(a[[1, 2, 3, 4]], b[[2, 1, 4, 3]], atol=1e-12)


def test_round_bf16_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -0.3])
    r = round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -7 and r[3] == 1.0 + 2 ** -6
    ref = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(r, ref)
