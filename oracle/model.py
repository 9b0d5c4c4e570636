"""Llama-style decoder forward in fp64 numpy.

Test infrastructure only (see oracle/__init__.py).

The paper names its models (llama-2-chat 7B / 70B, Sec. 5.1) but does not
restate their architecture; the forward below is the public Llama-2 decoder:

    x = E[tok]
    per layer:  a = RMSNorm(x; g_attn)
                q, k, v = a Wq^T, a Wk^T, a Wv^T        (no bias)
                q, k <- RoPE(q, k; position)             (rotate-half pairing)
                o = causal softmax(q k^T / sqrt(hd)) v   (GQA: q-head j reads kv-head j // (Hq/Hkv))
                x = x + o Wo^T
                m = RMSNorm(x; g_mlp)
                x = x + (SiLU(m Wg^T) * (m Wu^T)) Wd^T
    e = RMSNorm(x; g_final)                              (the "final embedding" of Eq. 3)
    logits = e W_lm^T

`forward_full` recomputes the whole prefix on every call (the definitional mode:
no cache, so no cache bug can hide in it).  `CachedForward` keeps plain K/V
arrays and is only trusted because a test shows it equals `forward_full`.

The paper fixes no numeric value for a forward pass ("parity unpinned" against
the paper); it is pinned to library routines and invariants in
tests/test_oracle_model.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np


@dataclass
class LayerWeights:
    wq: np.ndarray          # [Hq*hd, d]
    wk: np.ndarray          # [Hkv*hd, d]
    wv: np.ndarray          # [Hkv*hd, d]
    wo: np.ndarray          # [d, Hq*hd]
    w_gate: np.ndarray      # [ffn, d]
    w_up: np.ndarray        # [ffn, d]
    w_down: np.ndarray      # [d, ffn]
    norm_attn: np.ndarray   # [d]
    norm_mlp: np.ndarray    # [d]


@dataclass
class ModelWeights:
    n_heads: int
    n_kv_heads: int
    head_dim: int
    tok_emb: np.ndarray     # [V, d]
    lm_head: np.ndarray     # [V, d]
    final_norm: np.ndarray  # [d]
    layers: List[LayerWeights] = field(default_factory=list)
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def d_model(self) -> int:
        return self.tok_emb.shape[1]

    @property
    def vocab(self) -> int:
        return self.tok_emb.shape[0]


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x * g / sqrt(mean(x^2) + eps), row-wise."""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(g)


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.  v: [T, H, hd]; pos: [T] positions.
    Pair (i, i + hd/2) is rotated by the angle pos * theta**(-2i/hd)."""
    v = _f64(v)
    hd = v.shape[-1]
    half = hd // 2
    freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)      # [half]
    ang = _f64(pos)[:, None] * freq[None, :]                               # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """Causal softmax attention with grouped queries.

    q: [Tq, Hq, hd] at absolute positions q_pos[Tq]; k, v: [Tk, Hkv, hd] hold
    positions 0..Tk-1.  Query at position s sees keys 0..s.  Returns [Tq, Hq*hd].
    """
    tq, hq, hd = q.shape
    tk, hkv, _ = k.shape
    group = hq // hkv
    out = np.zeros((tq, hq, hd), dtype=np.float64)
    key_pos = np.arange(tk)
    for j in range(hq):
        g = j // group
        s = (q[:, j, :] @ k[:, g, :].T) / np.sqrt(float(hd))              # [Tq, Tk]
        s = np.where(key_pos[None, :] <= np.asarray(q_pos)[:, None], s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        w = np.exp(s)
        w = w / w.sum(axis=-1, keepdims=True)
        out[:, j, :] = w @ v[:, g, :]
    return out.reshape(tq, hq * hd)


def decoder_layer(w: ModelWeights, lw: LayerWeights, x: np.ndarray) -> np.ndarray:
    """One decoder layer over a whole sequence with no cache: x [T, d] holds the residual
    stream of positions 0..T-1 and the result is the residual stream after the layer."""
    t = x.shape[0]
    pos = np.arange(t)
    hq, hkv, hd = w.n_heads, w.n_kv_heads, w.head_dim
    a = rmsnorm(x, lw.norm_attn, w.rms_eps)
    q = (a @ _f64(lw.wq).T).reshape(t, hq, hd)
    k = (a @ _f64(lw.wk).T).reshape(t, hkv, hd)
    v = (a @ _f64(lw.wv).T).reshape(t, hkv, hd)
    q = rope(q, pos, w.rope_theta)
    k = rope(k, pos, w.rope_theta)
    o = attention(q, k, v, pos)
    x = x + o @ _f64(lw.wo).T
    m = rmsnorm(x, lw.norm_mlp, w.rms_eps)
    return x + (silu(m @ _f64(lw.w_gate).T) * (m @ _f64(lw.w_up).T)) @ _f64(lw.w_down).T


def final_logits(w: ModelWeights, x: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """(logits, e) of the residual rows x: e = final RMSNorm, logits = e W_lm^T."""
    e = rmsnorm(x, w.final_norm, w.rms_eps)
    return e @ _f64(w.lm_head).T, e


def forward_full(w: ModelWeights, tokens) -> tuple[np.ndarray, np.ndarray]:
    """Forward over the whole sequence with no cache.

    Returns (logits [T, V], final hidden e [T, d]); row t is conditioned on
    tokens[0..t].
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    x = _f64(w.tok_emb)[tokens]
    for lw in w.layers:
        x = decoder_layer(w, lw, x)
    return final_logits(w, x)


class CachedForward:
    """The same forward with plain per-layer K/V arrays (positions 0..len-1).

    `extend(tokens)` ingests tokens at positions len..len+T-1 and returns their
    (logits, hidden) rows; `truncate(n)` drops every position >= n.
    """

    def __init__(self, w: ModelWeights):
        self.w = w
        self.len = 0
        self.k = [np.zeros((0, w.n_kv_heads, w.head_dim)) for _ in w.layers]
        self.v = [np.zeros((0, w.n_kv_heads, w.head_dim)) for _ in w.layers]

    def truncate(self, n: int) -> None:
        assert 0 <= n <= self.len
        self.len = n
        self.k = [k[:n] for k in self.k]
        self.v = [v[:n] for v in self.v]

    def extend(self, tokens) -> tuple[np.ndarray, np.ndarray]:
        w = self.w
        tokens = np.asarray(tokens, dtype=np.int64)
        t = tokens.shape[0]
        pos = np.arange(self.len, self.len + t)
        hq, hkv, hd = w.n_heads, w.n_kv_heads, w.head_dim
        x = _f64(w.tok_emb)[tokens]
        for li, lw in enumerate(w.layers):
            a = rmsnorm(x, lw.norm_attn, w.rms_eps)
            q = rope((a @ _f64(lw.wq).T).reshape(t, hq, hd), pos, w.rope_theta)
            k = rope((a @ _f64(lw.wk).T).reshape(t, hkv, hd), pos, w.rope_theta)
            v = (a @ _f64(lw.wv).T).reshape(t, hkv, hd)
            self.k[li] = np.concatenate([self.k[li], k], axis=0)
            self.v[li] = np.concatenate([self.v[li], v], axis=0)
            o = attention(q, self.k[li], self.v[li], pos)
            x = x + o @ _f64(lw.wo).T
            m = rmsnorm(x, lw.norm_mlp, w.rms_eps)
            x = x + (silu(m @ _f64(lw.w_gate).T) * (m @ _f64(lw.w_up).T)) @ _f64(lw.w_down).T
        self.len += t
        e = rmsnorm(x, w.final_norm, w.rms_eps)
        return e @ _f64(w.lm_head).T, e
