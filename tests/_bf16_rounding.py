"""The oracle's decoder layer with the activations rounded to bfloat16 at the points where a bf16
model stores them, and nowhere else.  Test infrastructure: it composes oracle.model's own functions
(rmsnorm's formula, rope, silu, the attention definition) in fp64 and shares nothing with the HIP
sources.

What it is for: the tolerance on bf16 logits (2e-2, row-wise max-norm) is a statement about kernels,
not about bf16 storage.  A path that keeps a bf16 KV cache and feeds bf16 operands to its products
differs from the fp64 definition by the rounding of its stored activations, and through a deep
random-init stack those perturbations add up.  Comparing the HIP path with THIS forward (same
roundings, everything else fp64) separates the two: what is left is the kernels' own error
(fp32 accumulation order, fast exponentials), which must stay inside the tolerance at any depth.

Rounding points per decoder layer (R = round to nearest even bf16):
  1. the RMSNorm output that feeds q|k|v and the one that feeds gate|up.  A launch with few rows
     ("fused") stores R(x * gain) and applies the row's factor r = 1/sqrt(mean(x^2) + eps) to the sums
     of the product that consumes it; otherwise R((x * r) * gain) is stored;
  2. q and k after the rotary embedding, and v (the KV cache is bf16);
  3. the softmax weights exp(s - m) as the operand of the value product, m being the maximum over
     the visible keys of the row's 64-key block (key-split launches: every block on its own, merged
     by their maxima and unrounded sums) or the running maximum (prompt pass, blocks in order);
  4. the attention output;
  5. silu(gate) * up.
The residual stream, every sum, the softmax statistics and the logits are not rounded.

`dtype` selects the arithmetic everything else runs in.  float64 gives the reference.  float32 (every
intermediate array held in fp32, products through numpy's fp32 matrix multiply) is a second, plain
implementation of the same roundings: how far IT lands from the float64 one is what fp32 arithmetic
costs on this model, independent of any GPU kernel (a value that differs by one fp32 ulp before a
bf16 rounding can land on the other neighbour, and random-init layers amplify that), and is the
yardstick for the HIP path's distance from the float64 one.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np

from oracle.model import LayerWeights, ModelWeights, rope, silu

KEY_BLOCK = 64


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Nearest-even bfloat16 of every element, returned as fp64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def identity(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def _blocked_attention(q, k, v, q_pos, full: bool, rnd: Callable, rnd_out: Callable) -> np.ndarray:
    """oracle.model.attention with the softmax weights rounded per 64-key block (point 3) and
    the output rounded (point 4).  q [Tq, Hq, hd]; k, v [Tk, Hkv, hd] hold positions 0..Tk-1.
    Runs in the dtype of q."""
    tq, hq, hd = q.shape
    tk, hkv, _ = k.shape
    dt = q.dtype.type
    group = hq // hkv
    out = np.zeros((tq, hq, hd), dtype=dt)
    nblk = (tk + KEY_BLOCK - 1) // KEY_BLOCK
    for j in range(hq):
        g = j // group
        s_all = (q[:, j, :] @ k[:, g, :].T) / dt(np.sqrt(float(hd)))                 # [Tq, Tk]
        for t in range(tq):
            lim = int(q_pos[t])
            ms, ls, os_ = [], [], []
            m_run, l_run, o_run = dt(-np.inf), dt(0.0), np.zeros(hd, dtype=dt)
            for b in range(nblk):
                lo, hi = b * KEY_BLOCK, min((b + 1) * KEY_BLOCK, tk, lim + 1)
                if hi <= lo:
                    break
                s = s_all[t, lo:hi]
                if full:                                   # online softmax over the blocks in order
                    m_new = max(m_run, s.max())
                    alpha = np.exp(m_run - m_new) if np.isfinite(m_run) else dt(0.0)
                    e = np.exp(s - m_new)
                    l_run = l_run * alpha + e.sum()
                    o_run = o_run * alpha + rnd(e) @ v[lo:hi, g, :]
                    m_run = m_new
                else:                                      # every block on its own, merged below
                    m_b = s.max()
                    e = np.exp(s - m_b)
                    ms.append(m_b)
                    ls.append(e.sum())
                    os_.append(rnd(e) @ v[lo:hi, g, :])
            if full:
                out[t, j, :] = o_run / l_run
            else:
                mx = max(ms)
                wgt = np.exp(np.asarray(ms, dtype=dt) - mx)
                num = sum(wb * ob for wb, ob in zip(wgt, os_))
                den = np.dot(wgt, np.asarray(ls, dtype=dt))
                out[t, j, :] = num / den
    return rnd_out(out.reshape(tq, hq * hd))


class Chunk:
    """Rows of one launch: consecutive positions start .. start + T - 1 of the sequence."""

    def __init__(self, x: np.ndarray, start: int, fused: bool, full_attn: bool):
        self.x = x                                        # residual stream [T, d]
        self.pos = np.arange(start, start + self.x.shape[0])
        self.fused = fused
        self.full_attn = full_attn


class RoundedDecoder:
    """A sequence ingested as chunks (launches), layer by layer, so that a model whose layers are
    streamed one at a time needs a single sweep.  `rnd` = bf16_round gives the emulation,
    `identity` must reproduce oracle.model.forward_full (that is its CPU pin)."""

    def __init__(self, w: ModelWeights, tokens: Sequence[int], chunk_rows: Sequence[int], fused: Sequence[bool],
                 full_attn: Sequence[bool], rnd: Callable = bf16_round, skip: Sequence[str] = (),
                 dtype=np.float64):
        """skip: rounding points left out, of "norm", "qkv", "softmax", "attn", "act" (to see what each
        is worth).  dtype: the arithmetic (see the module text); the layers handed to layer() should
        hold their matrices in it, or every product converts them."""
        assert sum(chunk_rows) == len(tokens)
        self.w, self.dt = w, np.dtype(dtype).type
        cast = lambda fn: (lambda a: fn(a).astype(self.dt, copy=False))
        self.r = {name: cast(identity if name in skip else rnd) for name in ("norm", "qkv", "softmax", "attn", "act")}
        emb = np.asarray(w.tok_emb)[np.asarray(tokens, dtype=np.int64)].astype(self.dt)
        self.chunks: List[Chunk] = []
        s = 0
        for rows, fu, fa in zip(chunk_rows, fused, full_attn):
            self.chunks.append(Chunk(emb[s:s + rows], s, fu, fa))
            s += rows
        self.layers_done = 0
        self._lm = None

    def _norm_in(self, c: Chunk, gain: np.ndarray, deferred: bool):
        """(stored rows, factor the consumer applies to its sums)."""
        w, rnd, dt = self.w, self.r["norm"], self.dt
        r = dt(1.0) / np.sqrt(np.mean(c.x * c.x, axis=-1, keepdims=True) + dt(w.rms_eps))
        g = np.asarray(gain, dtype=dt)
        if deferred:
            return rnd(c.x * g), r
        return rnd((c.x * r) * g), dt(1.0)

    def layer(self, lw: LayerWeights) -> None:
        """Advance every chunk through one decoder layer."""
        w, rnd, dt = self.w, self.r["qkv"], self.dt
        hq, hkv, hd = w.n_heads, w.n_kv_heads, w.head_dim
        f = lambda a: np.asarray(a, dtype=dt)
        k_all = np.zeros((0, hkv, hd), dtype=dt)
        v_all = np.zeros((0, hkv, hd), dtype=dt)
        first = self.layers_done == 0
        for c in self.chunks:
            t = c.x.shape[0]
            # the attention norm's rows come from the embedding kernel (first layer) or from the
            # previous layer's down projection: only the latter defers the row factor
            a, r = self._norm_in(c, lw.norm_attn, c.fused and not first)
            q = rnd(rope(((a @ f(lw.wq).T) * r).reshape(t, hq, hd), c.pos, w.rope_theta))
            k = rnd(rope(((a @ f(lw.wk).T) * r).reshape(t, hkv, hd), c.pos, w.rope_theta))
            v = rnd(((a @ f(lw.wv).T) * r).reshape(t, hkv, hd))
            k_all = np.concatenate([k_all, k], axis=0)
            v_all = np.concatenate([v_all, v], axis=0)
            o = _blocked_attention(q, k_all, v_all, c.pos, c.full_attn, self.r["softmax"], self.r["attn"])
            c.x = c.x + o @ f(lw.wo).T
            m, r = self._norm_in(c, lw.norm_mlp, c.fused)
            act = self.r["act"](silu((m @ f(lw.w_gate).T) * r) * ((m @ f(lw.w_up).T) * r))
            c.x = c.x + act @ f(lw.w_down).T
        self.layers_done += 1

    def logits(self, chunk: int = -1) -> np.ndarray:
        """Logits of a chunk's rows after the layers done so far (final RMSNorm, stored rounded)."""
        c = self.chunks[chunk]
        e, _ = self._norm_in(c, self.w.final_norm, False)
        if self._lm is None:
            self._lm = np.asarray(self.w.lm_head, dtype=self.dt)
        return (e @ self._lm.T).astype(np.float64)
