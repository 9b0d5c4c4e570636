"""Test helpers: hand the synthetic tensors to the CPU oracle as numpy arrays."""
import numpy as np
import torch

from oracle.head import HeadWeights
from oracle.model import LayerWeights, ModelWeights


def _np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def oracle_model(m: dict) -> ModelWeights:
    """Split the stacked q|k|v and gate|up matrices into the separate projections
    the oracle's definition uses."""
    s = m["shape"]
    layers = []
    for lay in m["layers"]:
        wqkv, wgu = _np(lay["wqkv"]), _np(lay["w_gate_up"])
        layers.append(LayerWeights(
            wq=wqkv[: s.n_q], wk=wqkv[s.n_q: s.n_q + s.n_kv], wv=wqkv[s.n_q + s.n_kv:],
            wo=_np(lay["wo"]), w_gate=wgu[: s.d_ffn], w_up=wgu[s.d_ffn:], w_down=_np(lay["w_down"]),
            norm_attn=_np(lay["norm_attn"]), norm_mlp=_np(lay["norm_mlp"])))
    return ModelWeights(n_heads=s.n_heads, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                        tok_emb=_np(m["tok_emb"]), lm_head=_np(m["lm_head"]), final_norm=_np(m["final_norm"]),
                        layers=layers, rope_theta=s.rope_theta, rms_eps=s.rms_eps)


def oracle_head(h: dict) -> HeadWeights:
    return HeadWeights(W=[_np(w) for w in h["W"]], b=[_np(b) for b in h["b"]], residual=h["residual"])


class StreamedLayers:
    """Layers of a synthetic model handed to the oracle one at a time: each layer's matrices are
    converted to fp64 on the device they live on and copied to the host when the oracle's forward
    reaches that layer (a 70B-shaped layer is 6.9 GB in fp64; eighty of them do not fit in host memory).
    The host copies live in pinned buffers that the next layer overwrites, so a layer's arrays are
    valid only until the iterator is advanced (a forward pass is done with a layer by then).
    `progress(i, n)` is called before layer i is fetched.  `dtype`: the arrays' type (torch.float64 for
    the oracle; torch.float32 holds bf16 weights exactly too, for an fp32 re-run of the same forward)."""

    _MATS = ("wqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp")

    def __init__(self, m: dict, progress=None, dtype=torch.float64):
        self.m = m
        self.progress = progress
        self.dtype = dtype

    def __len__(self):
        return len(self.m["layers"])

    def __iter__(self):
        s = self.m["shape"]
        bufs = {}
        n = len(self.m["layers"])
        for i, lay in enumerate(self.m["layers"]):
            if self.progress is not None:
                self.progress(i, n)
            a = {}
            for name in self._MATS:
                src = lay[name].detach()
                if src.is_cuda:
                    if name not in bufs:
                        bufs[name] = torch.empty(src.shape, dtype=self.dtype, pin_memory=True)
                    bufs[name].copy_(src.to(self.dtype))
                    a[name] = bufs[name].numpy()
                else:
                    a[name] = src.to(self.dtype).numpy()
            wqkv, wgu = a["wqkv"], a["w_gate_up"]
            yield LayerWeights(
                wq=wqkv[: s.n_q], wk=wqkv[s.n_q: s.n_q + s.n_kv], wv=wqkv[s.n_q + s.n_kv:],
                wo=a["wo"], w_gate=wgu[: s.d_ffn], w_up=wgu[s.d_ffn:], w_down=a["w_down"],
                norm_attn=a["norm_attn"], norm_mlp=a["norm_mlp"])


def oracle_model_streamed(m: dict, progress=None) -> ModelWeights:
    s = m["shape"]
    f = lambda t: t.detach().to(torch.float64).cpu().numpy()
    return ModelWeights(n_heads=s.n_heads, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, tok_emb=f(m["tok_emb"]),
                        lm_head=f(m["lm_head"]), final_norm=f(m["final_norm"]), layers=StreamedLayers(m, progress),
                        rope_theta=s.rope_theta, rms_eps=s.rms_eps)
