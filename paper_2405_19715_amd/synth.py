"""Seeded synthetic inputs: model shapes, random-init weights, prompts, logits.

This module draws random numbers and lays them out; it holds none of the
method's arithmetic (no forward pass, no softmax, no sampling), so the HIP path
and the CPU checker can both be fed from it without sharing any computation.

The paper measured on dataset prompts with trained llama-2-chat weights
(Sec. 5.1, Appendix D.1); neither exists here.  These inputs take that
workload's shapes (Llama-2 dimensions, vocab 32000, bf16, batch 1) and stand in
for it: weights are N(0, 0.02), prompts are uniform random token ids.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import torch


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def n_q(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def n_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def layer_params(self) -> int:
        d = self.d_model
        return (self.n_q + 2 * self.n_kv) * d + d * self.n_q + 3 * self.d_ffn * d

    def streamed_params(self) -> int:
        """Weights one forward pass reads: every layer plus the LM head."""
        return self.n_layers * self.layer_params() + self.vocab * self.d_model


# Shapes of the workloads (tiny fp32 pair; 7B / 1.1B-shaped pair; 70B / 7B-shaped pair).
TINY_TARGET = ModelShape(2, 256, 4, 4, 64, 688, 1024)
TINY_DRAFT = replace(TINY_TARGET, n_layers=1)
LLAMA_1B = ModelShape(22, 2048, 32, 4, 64, 5632, 32000)
LLAMA_7B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
LLAMA_70B = ModelShape(80, 8192, 64, 8, 128, 28672, 32000)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std: float, g: torch.Generator, device, dtype) -> torch.Tensor:
    """N(0, std) drawn in fp32 then rounded to dtype.  Drawn in row blocks so a
    multi-GB bf16 tensor never needs an fp32 twin of the same size."""
    out = torch.empty(shape, device=device, dtype=dtype)
    rows = shape[0]
    cols = int(math.prod(shape[1:])) if len(shape) > 1 else 1
    step = max(1, (64 << 20) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g, device=device, dtype=torch.float32)
        out[r0:r1] = (blk * std).to(dtype)
    return out


def make_model(shape: ModelShape, seed: int, device="cpu", dtype=torch.float32, std: float = 0.02) -> Dict:
    """Random-init decoder weights.  Matrices are [out, in] row-major; q|k|v and
    gate|up are stored stacked along the output dimension."""
    g = _gen(seed, device)
    d = shape.d_model
    m = dict(shape=shape, dtype=dtype,
             tok_emb=_normal((shape.vocab, d), std, g, device, dtype),
             lm_head=_normal((shape.vocab, d), std, g, device, dtype),
             final_norm=torch.ones(d, device=device, dtype=dtype),
             layers=[])
    for _ in range(shape.n_layers):
        m["layers"].append(dict(
            wqkv=_normal((shape.n_q + 2 * shape.n_kv, d), std, g, device, dtype),
            wo=_normal((d, shape.n_q), std, g, device, dtype),
            w_gate_up=_normal((2 * shape.d_ffn, d), std, g, device, dtype),
            w_down=_normal((d, shape.d_ffn), std, g, device, dtype),
            norm_attn=torch.ones(d, device=device, dtype=dtype),
            norm_mlp=torch.ones(d, device=device, dtype=dtype)))
    return m


def make_perturbed_draft(target: Dict, n_layers: int, seed: int, std: float = 0.005) -> Dict:
    """Draft = the target's first n_layers with N(0, std) added to the layer
    matrices; embedding, LM head and final norm are the target's own buffers."""
    shape = replace(target["shape"], n_layers=n_layers)
    dev, dt = target["tok_emb"].device, target["dtype"]
    g = _gen(seed, dev)
    m = dict(shape=shape, dtype=dt, tok_emb=target["tok_emb"], lm_head=target["lm_head"],
             final_norm=target["final_norm"], layers=[])
    for li in range(n_layers):
        src = target["layers"][li]
        lay = {}
        for name in ("wqkv", "wo", "w_gate_up", "w_down"):
            noise = torch.randn(src[name].shape, generator=g, device=dev, dtype=torch.float32) * std
            lay[name] = (src[name].float() + noise).to(dt)
        lay["norm_attn"] = src["norm_attn"].clone()
        lay["norm_mlp"] = src["norm_mlp"].clone()
        m["layers"].append(lay)
    return m


def damp_tail(model: Dict, first: int, gain: float) -> None:
    """Scale, in place, the two matrices that write into the residual stream (wo, w_down)
    of layers first.. by `gain`.  With gain < 1 those layers move the final hidden state
    only a little, so a draft made of the layers before them (make_perturbed_draft) stays
    aligned with the full model: the recipe for a pair whose acceptance rate is tunable
    without trained weights."""
    for lay in model["layers"][first:]:
        for name in ("wo", "w_down"):
            lay[name].mul_(gain)


def align_narrow_draft(target: Dict, draft: Dict, layer_gain: float, extra_gain: float) -> None:
    """Make, in place, a pair of DIFFERENT widths whose next-token distributions agree to a
    tunable degree without trained weights (d_draft < d_target, same vocabulary):
      * every layer of both models is damped by `layer_gain` (damp_tail from layer 0), so the
        final hidden state of a row is close to the embedding of its input token and both
        models are essentially bigram tables, while all weights are still streamed and multiplied;
      * the draft's embedding and LM head become the first d_draft columns of the target's, so its
        logits are the part of the target's logit sum that runs over those columns;
      * the remaining columns of the target's LM head are scaled by `extra_gain`: they add a
        per-token logit shift of about N(0, (0.02 extra_gain)^2 (d_target - d_draft)) that the
        draft cannot see.  With sigma that standard deviation, the acceptance rate
        sum_v min(p_v, q_v) is about 2 Phi(-sigma / 2) for a large vocabulary."""
    dd = draft["tok_emb"].shape[1]
    damp_tail(target, 0, layer_gain)
    damp_tail(draft, 0, layer_gain)
    draft["tok_emb"] = target["tok_emb"][:, :dd].contiguous()
    draft["lm_head"] = target["lm_head"][:, :dd].contiguous()
    target["lm_head"][:, dd:].mul_(extra_gain)


def mark_hard_tokens(target: Dict, draft: Dict, frac: float, marker: float, c: float, seed: int) -> torch.Tensor:
    """Give the pair a marked subset H of the vocabulary (a fraction `frac` of the token ids) on
    which the draft's output layer disagrees with the target's: the draft gets its own LM head
    whose rows in H carry extra N(0, c^2 / d) noise (a logit shift of about N(0, c^2) per
    context), and the shared embedding of every token in H gets `marker` times one fixed unit
    vector, so that the final embedding of a row whose input token is in H says so.  Whether a
    drafted token will be accepted then depends on the token, and the token is visible to an
    acceptance-prediction head.  Returns the boolean mask of H."""
    dev, dt = target["tok_emb"].device, target["dtype"]
    V, d = target["tok_emb"].shape
    g = _gen(seed, dev)
    hard = torch.rand((V,), generator=g, device=dev) < frac
    u = torch.randn((d,), generator=g, device=dev, dtype=torch.float32)
    u = u / u.norm()
    emb = target["tok_emb"].float()
    emb[hard] += marker * u
    target["tok_emb"].copy_(emb.to(dt))
    draft["tok_emb"] = target["tok_emb"]
    lm = target["lm_head"].float()
    noise = torch.randn((int(hard.sum()), d), generator=g, device=dev, dtype=torch.float32) * (c / math.sqrt(d))
    lm[hard] += noise
    draft["lm_head"] = lm.to(dt).contiguous()
    return hard


def make_head(dims: List[int], seed: int, device="cpu", dtype=torch.float32, residual: bool = False,
              out_bias: float = 1.386, std: float = 0.02) -> Dict:
    """Acceptance-head weights: len(dims)-1 layers, dims[-1] == 1.  The output bias
    logit(0.8) = 1.386 makes the mean predicted acceptance about 0.8."""
    assert dims[-1] == 1
    g = _gen(seed, device)
    W, b = [], []
    for j in range(len(dims) - 1):
        W.append(_normal((dims[j + 1], dims[j]), std, g, device, dtype))
        b.append(torch.zeros(dims[j + 1], device=device, dtype=dtype))
    b[-1] = torch.full((1,), out_bias, device=device, dtype=dtype)
    return dict(dims=list(dims), W=W, b=b, residual=bool(residual), dtype=dtype)


def make_prompt(n: int, vocab: int, seed: int) -> List[int]:
    g = _gen(seed, "cpu")
    return torch.randint(0, vocab, (n,), generator=g).tolist()


def make_accept_logits(batch: int, k: int, vocab: int, seed: int, device="cpu",
                       target_std: float = 2.0, noise_std: float = 0.5):
    """Logits for the isolated accept / resample case: target rows ~ N(0, 2^2) for
    K+1 positions; draft rows = the first K target rows + N(0, 0.5^2).  fp32."""
    g = _gen(seed, device)
    p = torch.randn((batch, k + 1, vocab), generator=g, device=device) * target_std
    q = p[:, :k, :] + torch.randn((batch, k, vocab), generator=g, device=device) * noise_std
    return p.contiguous(), q.contiguous()
