"""Pins for oracle/model.py.  The paper prints no forward-pass values, so the
forward is pinned to library routines (torch's scaled_dot_product_attention,
rms_norm, silu, linear; complex multiplication for the rotary embedding) and to
invariants a wrong sign, index or transposition would break."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import model as M
from paper_2405_19715_amd import synth
from tests._util import oracle_model

SHAPE_GQA = synth.ModelShape(n_layers=2, d_model=48, n_heads=6, n_kv_heads=2, head_dim=8, d_ffn=80, vocab=61)
SHAPE_MHA = synth.ModelShape(n_layers=2, d_model=32, n_heads=4, n_kv_heads=4, head_dim=8, d_ffn=56, vocab=50)


def _model(shape, seed=0, std=0.3):
    m = synth.make_model(shape, seed, dtype=torch.float64, std=std)
    g = torch.Generator().manual_seed(seed + 100)
    # non-trivial norm gains so a dropped gain is caught
    m["final_norm"] = 1 + 0.2 * torch.randn(shape.d_model, generator=g, dtype=torch.float64)
    for lay in m["layers"]:
        lay["norm_attn"] = 1 + 0.2 * torch.randn(shape.d_model, generator=g, dtype=torch.float64)
        lay["norm_mlp"] = 1 + 0.2 * torch.randn(shape.d_model, generator=g, dtype=torch.float64)
    return m


def _torch_forward(m, tokens):
    """The same decoder written with torch library routines only."""
    s = m["shape"]
    t = len(tokens)
    x = m["tok_emb"][torch.tensor(tokens)]
    half = s.head_dim // 2
    inv = s.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2 / s.head_dim)
    rot = torch.polar(torch.ones(t, half, dtype=torch.float64), torch.arange(t, dtype=torch.float64)[:, None] * inv)

    def rope(v):                                   # [T, H, hd]; pair (i, i+half) as one complex number
        z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for lay in m["layers"]:
        a = F.rms_norm(x, (s.d_model,), lay["norm_attn"], s.rms_eps)
        qkv = F.linear(a, lay["wqkv"])
        q = rope(qkv[:, : s.n_q].reshape(t, s.n_heads, s.head_dim))
        k = rope(qkv[:, s.n_q: s.n_q + s.n_kv].reshape(t, s.n_kv_heads, s.head_dim))
        v = qkv[:, s.n_q + s.n_kv:].reshape(t, s.n_kv_heads, s.head_dim)
        rep = s.n_heads // s.n_kv_heads
        k, v = k.repeat_interleave(rep, dim=1), v.repeat_interleave(rep, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        x = x + F.linear(o.transpose(0, 1).reshape(t, s.n_q), lay["wo"])
        mm = F.rms_norm(x, (s.d_model,), lay["norm_mlp"], s.rms_eps)
        gu = F.linear(mm, lay["w_gate_up"])
        x = x + F.linear(F.silu(gu[:, : s.d_ffn]) * gu[:, s.d_ffn:], lay["w_down"])
    e = F.rms_norm(x, (s.d_model,), m["final_norm"], s.rms_eps)
    return F.linear(e, m["lm_head"]).numpy(), e.numpy()


def test_forward_matches_torch_library_routines():
    for shape in (SHAPE_GQA, SHAPE_MHA):
        m = _model(shape)
        toks = synth.make_prompt(13, shape.vocab, 3)
        logits, hid = M.forward_full(oracle_model(m), toks)
        want_logits, want_hid = _torch_forward(m, toks)
        np.testing.assert_allclose(logits, want_logits, rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(hid, want_hid, rtol=1e-9, atol=1e-10)


def test_rope_position_zero_is_identity_and_is_a_rotation():
    rng = np.random.default_rng(0)
    v = rng.normal(size=(3, 2, 16))
    np.testing.assert_allclose(M.rope(v, np.zeros(3), 10000.0), v, atol=0)
    r = M.rope(v, np.array([5, 17, 400]), 10000.0)
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=(1, 1, 32)), rng.normal(size=(1, 1, 32))
    def score(m, n):
        return float(np.sum(M.rope(q, np.array([m]), 10000.0) * M.rope(k, np.array([n]), 10000.0)))
    assert abs(score(9, 4) - score(105, 100)) < 1e-10
    assert abs(score(9, 4) - score(4, 9)) > 1e-6       # direction matters
    # first pair rotates by exactly pos radians (frequency theta^0 = 1)
    e0 = np.zeros((1, 1, 32)); e0[0, 0, 0] = 1.0
    r = M.rope(e0, np.array([1]), 10000.0)[0, 0]
    assert abs(r[0] - np.cos(1.0)) < 1e-15 and abs(r[16] - np.sin(1.0)) < 1e-15


def test_rmsnorm_of_constant_vector():
    x = np.full((1, 10), 3.0)
    g = np.arange(1, 11, dtype=float)
    np.testing.assert_allclose(M.rmsnorm(x, g, 0.0), g[None, :], rtol=1e-15)
    np.testing.assert_allclose(M.rmsnorm(-x, g, 0.0), -g[None, :], rtol=1e-15)


def test_causality_and_prefix_consistency():
    m = oracle_model(_model(SHAPE_GQA, seed=2))
    toks = synth.make_prompt(12, SHAPE_GQA.vocab, 5)
    full, _ = M.forward_full(m, toks)
    for t in (1, 5, 11):
        part, _ = M.forward_full(m, toks[:t])
        np.testing.assert_allclose(part, full[:t], rtol=1e-10, atol=1e-12)
    changed = list(toks); changed[7] = (changed[7] + 1) % SHAPE_GQA.vocab
    other, _ = M.forward_full(m, changed)
    np.testing.assert_allclose(other[:7], full[:7], rtol=1e-10, atol=1e-12)
    assert np.abs(other[7:] - full[7:]).max() > 1e-6


def test_cached_forward_equals_full_recompute_with_rollback():
    m = oracle_model(_model(SHAPE_GQA, seed=3))
    toks = synth.make_prompt(15, SHAPE_GQA.vocab, 6)
    full, full_h = M.forward_full(m, toks)
    c = M.CachedForward(m)
    a, ah = c.extend(toks[:6])
    np.testing.assert_allclose(a, full[:6], rtol=1e-10, atol=1e-12)
    c.extend([1, 2, 3, 4])                       # speculative rows that get rolled back
    c.truncate(6)
    b, bh = c.extend(toks[6:])
    np.testing.assert_allclose(b, full[6:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bh, full_h[6:], rtol=1e-10, atol=1e-12)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    mg = _model(SHAPE_GQA, seed=4)
    s = SHAPE_GQA
    og = oracle_model(mg)
    rep = s.n_heads // s.n_kv_heads
    import copy
    om = copy.deepcopy(og)
    om.n_kv_heads = s.n_heads
    for lw in om.layers:
        lw.wk = np.repeat(lw.wk.reshape(s.n_kv_heads, s.head_dim, -1), rep, axis=0).reshape(s.n_q, -1)
        lw.wv = np.repeat(lw.wv.reshape(s.n_kv_heads, s.head_dim, -1), rep, axis=0).reshape(s.n_q, -1)
    toks = synth.make_prompt(9, s.vocab, 7)
    np.testing.assert_allclose(M.forward_full(og, toks)[0], M.forward_full(om, toks)[0], rtol=1e-10, atol=1e-12)


def test_single_token_attention_is_identity_on_values():
    """One token, one layer, zero MLP: softmax over a single key is 1, so the
    layer output is x + Wo Wv rmsnorm(x), computable by hand."""
    shape = synth.ModelShape(1, 16, 2, 2, 8, 24, 11)
    m = _model(shape, seed=5)
    m["layers"][0]["w_down"].zero_()
    om = oracle_model(m)
    tok = 4
    x = om.tok_emb[tok]
    a = x / np.sqrt(np.mean(x * x) + om.rms_eps) * om.layers[0].norm_attn
    y = x + om.layers[0].wo @ (om.layers[0].wv @ a)
    e = y / np.sqrt(np.mean(y * y) + om.rms_eps) * om.final_norm
    logits, hid = M.forward_full(om, [tok])
    np.testing.assert_allclose(hid[0], e, rtol=1e-12)
    np.testing.assert_allclose(logits[0], om.lm_head @ e, rtol=1e-12)
