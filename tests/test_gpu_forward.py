"""Teacher-forced parity of the HIP forward pass (embedding, RMSNorm, skinny GEMMs,
rotary embedding + KV append, block attention with grouped queries, SwiGLU, LM
head) with the oracle's fp64 forward on the same tokens."""
import numpy as np
import pytest
import torch

from oracle.model import forward_full
from paper_2405_19715_amd import synth
from tests._util import oracle_model

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}     # row-wise max|diff| / max|logit|


def _cuda(m):
    out = dict(m)
    for k in ("tok_emb", "lm_head", "final_norm"):
        out[k] = m[k].cuda()
    out["layers"] = [{k: v.cuda() for k, v in lay.items()} for lay in m["layers"]]
    return out


def _row_err(got, want):
    return (np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()


def _forward_case(shape, dtype, n_tokens, chunks, seed=0, std=0.02):
    from paper_2405_19715_amd import binding as B
    m = synth.make_model(shape, seed, dtype=dtype, std=std)
    toks = synth.make_prompt(n_tokens, shape.vocab, seed + 1)
    want_logits, want_hid = forward_full(oracle_model(m), toks)
    mc = _cuda(m)
    ctx = B.Context(mc, mc, None, batch=1, max_seq=256, k_max=8)
    try:
        ctx.sd_prefill(0, toks[:1] + [0])          # P = 2: caches hold position 0 of a dummy; overwritten below
        got_l, got_h, start = [], [], 0
        for c in chunks:
            l, h = ctx.sd_forward(0, 0, start, toks[start:start + c], want_hidden=True)
            got_l.append(l.numpy()); got_h.append(h.numpy()); start += c
        assert start == n_tokens
        got_l, got_h = np.concatenate(got_l), np.concatenate(got_h)
        assert _row_err(got_l, want_logits) < TOL[dtype]
        assert _row_err(got_h, want_hid) < TOL[dtype]
        # rollback: re-ingest the tail after truncating the cache -> same rows again
        l2 = ctx.sd_forward(0, 0, n_tokens - 5, toks[n_tokens - 5:]).numpy()
        np.testing.assert_allclose(l2, got_l[-5:], rtol=0, atol=TOL[dtype] * np.abs(want_logits).max())
    finally:
        ctx.close()


def test_tiny_fp32_matches_oracle():
    _forward_case(synth.TINY_TARGET, torch.float32, 70, [32, 17, 1, 2, 9, 9])


def test_fp32_grouped_queries():
    shape = synth.ModelShape(2, 128, 8, 2, 32, 200, 300)
    _forward_case(shape, torch.float32, 40, [20, 1, 19], std=0.05)


@pytest.mark.parametrize("shape", [
    synth.ModelShape(2, 256, 2, 2, 128, 384, 2048),          # MHA, head_dim 128 (draft-like)
    synth.ModelShape(2, 512, 8, 1, 64, 640, 2048),           # 8:1 grouped queries, head_dim 64
    synth.ModelShape(2, 1024, 8, 1, 128, 1280, 2048),        # 8:1 grouped queries, head_dim 128 (target-like)
])
def test_bf16_matches_oracle(shape):
    # chunks: 17 rows with 8 query heads = 136 query vectors per KV head, then single rows
    _forward_case(shape, torch.bfloat16, 150, [32, 32, 32, 17, 17, 1, 2, 17], std=0.04)


# Widths that are multiples of 2048 send rows of up to 8 through the row-stripe GEMM, whose final sweep does the
# SiLU * up, both residual adds and the RMSNorm preparation (the consumers apply the rows' norm factors): chunks of
# every row count 1 .. 8 exercise each instantiation of the vector-ALU kernel, 9 .. 17 the matrix-core member of the
# family (same sweeps), 18 and more the tiled kernel with the separate small kernels, and the cache carries over
# between the kinds of pass.
@pytest.mark.parametrize("chunks", [[9, 1, 2, 3, 4, 5, 6, 7, 8, 17, 1, 8], [16, 15, 14, 13, 12, 11, 10, 9, 17, 18, 3]])
@pytest.mark.parametrize("shape", [
    synth.ModelShape(3, 2048, 16, 2, 128, 4096, 1024),       # q|k|v, o, gate|up, down all stripe-shaped (K = 2048 / 4096)
    synth.ModelShape(2, 2048, 32, 32, 64, 5632, 1024),       # down K = 5632 stays on the MFMA kernel (1.1B-like MLP)
    synth.ModelShape(2, 4096, 32, 4, 128, 2048 * 3, 512),    # 2 and 3 stripes per row
])
def test_bf16_fused_epilogues_match_oracle(shape, chunks):
    _forward_case(shape, torch.bfloat16, sum(chunks), chunks, std=0.02)


def test_bf16_long_context_many_key_splits():
    from paper_2405_19715_amd import binding as B
    shape = synth.ModelShape(1, 256, 4, 2, 64, 256, 512)
    m = synth.make_model(shape, 3, dtype=torch.bfloat16, std=0.05)
    toks = synth.make_prompt(700, shape.vocab, 4)
    want, _ = forward_full(oracle_model(m), toks)
    mc = _cuda(m)
    ctx = B.Context(mc, mc, None, batch=1, max_seq=1024, k_max=16)
    try:
        ctx.sd_prefill(0, toks[:1] + [0])
        start, rows = 0, []
        while start < 700:
            c = min(32, 700 - start)
            rows.append(ctx.sd_forward(0, 0, start, toks[start:start + c]).numpy())
            start += c
        got = np.concatenate(rows)
        assert _row_err(got, want) < TOL[torch.bfloat16]
    finally:
        ctx.close()


@pytest.mark.parametrize("shape,n,max_seq", [
    (synth.ModelShape(2, 512, 8, 1, 64, 640, 2048), 2, 256),        # one prompt row
    (synth.ModelShape(2, 512, 8, 1, 64, 640, 2048), 38, 256),       # less than one tile
    (synth.ModelShape(2, 256, 2, 2, 128, 384, 2048), 201, 256),     # MHA, head_dim 128, ragged tiles
    (synth.ModelShape(2, 1024, 8, 1, 128, 1280, 2048), 230, 256),   # 8:1 grouped queries, head_dim 128
    (synth.ModelShape(1, 256, 4, 2, 64, 256, 512), 1101, 1152),     # two prompt chunks (1024 + 76 rows)
    (synth.ModelShape(1, 128, 2, 1, 64, 128, 512), 8000, 8064),     # long context: 8 chunks, 126 key blocks to merge
])
def test_bf16_prompt_pass_matches_oracle(shape, n, max_seq):
    """The prompt pass (tiled large-M GEMM + unsplit causal attention) fills the KV cache
    with what the oracle's forward computes: the rows that follow, teacher-forced against
    that cache, must give the oracle's logits and final hidden states."""
    from paper_2405_19715_amd import binding as B
    m = synth.make_model(shape, 5, dtype=torch.bfloat16, std=0.04)
    tail = 6
    toks = synth.make_prompt(n + tail, shape.vocab, 6)
    want_logits, want_hid = forward_full(oracle_model(m), toks)
    mc = _cuda(m)
    ctx = B.Context(mc, mc, None, batch=1, max_seq=max_seq, k_max=8)
    try:
        ctx.sd_prefill(0, toks[:n])                 # caches now hold positions 0 .. n-2
        l, h = ctx.sd_forward(0, 0, n - 1, toks[n - 1:], want_hidden=True)
        assert _row_err(l.numpy(), want_logits[n - 1:]) < TOL[torch.bfloat16]
        assert _row_err(h.numpy(), want_hid[n - 1:]) < TOL[torch.bfloat16]
    finally:
        ctx.close()


def _last_rows_of_a_one_layer_model(m, toks, n):
    """Logits of rows n-1 .. of a ONE-layer model from the oracle's layer functions: every key and
    value depends on its own token only, so the last rows need no full T x T forward."""
    from oracle import model as OM
    shape = m["shape"]
    w = oracle_model(m)
    lw = w.layers[0]
    T = len(toks)
    pos = np.arange(T)
    x = w.tok_emb[np.asarray(toks)]
    a = OM.rmsnorm(x, lw.norm_attn, w.rms_eps)
    k = OM.rope((a @ lw.wk.T).reshape(T, shape.n_kv_heads, shape.head_dim), pos, w.rope_theta)
    v = (a @ lw.wv.T).reshape(T, shape.n_kv_heads, shape.head_dim)
    last = slice(n - 1, T)
    q = OM.rope((a[last] @ lw.wq.T).reshape(-1, shape.n_heads, shape.head_dim), pos[last], w.rope_theta)
    xl = x[last] + OM.attention(q, k, v, pos[last]) @ lw.wo.T
    h = OM.rmsnorm(xl, lw.norm_mlp, w.rms_eps)
    xl = xl + (OM.silu(h @ lw.w_gate.T) * (h @ lw.w_up.T)) @ lw.w_down.T
    return OM.rmsnorm(xl, w.final_norm, w.rms_eps) @ w.lm_head.T


def test_context_at_the_largest_cache_size():
    """max_seq = 32768, the most the attention kernels take (512 key blocks per row): 32700 prompt
    tokens through the prompt pass, then 6 teacher-forced rows whose attention merges 511 partials.
    The expected rows come from the oracle's layer functions applied to the last rows only (shown
    equal to its full forward on a short sequence first)."""
    from paper_2405_19715_amd import binding as B
    shape = synth.ModelShape(1, 128, 2, 1, 64, 128, 512)
    m = synth.make_model(shape, 8, dtype=torch.bfloat16, std=0.04)
    n, tail = 32700, 6
    toks = synth.make_prompt(n + tail, shape.vocab, 9)
    short = toks[:206]
    assert np.abs(_last_rows_of_a_one_layer_model(m, short, 200) - forward_full(oracle_model(m), short)[0][199:]).max() < 1e-12
    want = _last_rows_of_a_one_layer_model(m, toks, n)
    mc = _cuda(m)
    ctx = B.Context(mc, mc, None, batch=1, max_seq=32768, k_max=8)
    try:
        ctx.sd_prefill(0, toks[:n])
        got = ctx.sd_forward(0, 0, n - 1, toks[n - 1:]).numpy()
        assert _row_err(got, want) < TOL[torch.bfloat16]
        assert ctx.sd_seq_state(0)["P"] == n
    finally:
        ctx.close()
