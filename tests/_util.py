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
    reaches that layer (a 70B-shaped layer is 6.9 GB in fp64; eighty of them do not fit in host memory)."""

    def __init__(self, m: dict):
        self.m = m

    def __iter__(self):
        s = self.m["shape"]
        f = lambda t: t.detach().to(torch.float64).cpu().numpy()
        for i, lay in enumerate(self.m["layers"]):
            if i % 8 == 0 and len(self.m["layers"]) > 8:
                print(f"oracle: layer {i} of {len(self.m['layers'])}", flush=True)      # visible with pytest -s
            wqkv, wgu = f(lay["wqkv"]), f(lay["w_gate_up"])
            yield LayerWeights(
                wq=wqkv[: s.n_q], wk=wqkv[s.n_q: s.n_q + s.n_kv], wv=wqkv[s.n_q + s.n_kv:],
                wo=f(lay["wo"]), w_gate=wgu[: s.d_ffn], w_up=wgu[s.d_ffn:], w_down=f(lay["w_down"]),
                norm_attn=f(lay["norm_attn"]), norm_mlp=f(lay["norm_mlp"]))


def oracle_model_streamed(m: dict) -> ModelWeights:
    s = m["shape"]
    f = lambda t: t.detach().to(torch.float64).cpu().numpy()
    return ModelWeights(n_heads=s.n_heads, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim, tok_emb=f(m["tok_emb"]),
                        lm_head=f(m["lm_head"]), final_norm=f(m["final_norm"]), layers=StreamedLayers(m),
                        rope_theta=s.rope_theta, rms_eps=s.rms_eps)
