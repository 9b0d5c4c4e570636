"""ctypes binding of libspecdec.so: the same entry points as include/specdec.h, with
argument marshalling only (torch tensors -> device pointers, lists -> C arrays).
Every step of the path runs in the library's HIP kernels; nothing here computes.

Importing this module loads the library and raises if it has not been built
(`python -m paper_2405_19715_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspecdec.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2405_19715_amd.build`")
lib = C.CDLL(_LIB_PATH)

SD_OK, SD_EINVAL, SD_ENOMEM, SD_ERANGE, SD_ENONFINITE, SD_EDEVICE = 0, -1, -2, -3, -4, -5
SD_F32, SD_BF16 = 0, 1
SD_MAX_K = 32

_vpp = C.POINTER(C.c_void_p)


class sd_model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("wqkv", _vpp), ("wo", _vpp), ("w_gate_up", _vpp), ("w_down", _vpp),
                ("norm_attn", _vpp), ("norm_mlp", _vpp)]


class sd_head(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("residual", C.c_int32),
                ("dtype", C.c_int32), ("W", _vpp), ("b", _vpp)]


class sd_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("max_seq", C.c_int32), ("k_max", C.c_int32), ("hip_stream", C.c_void_p)]


class sd_params(C.Structure):
    _fields_ = [("h", C.c_float), ("temperature", C.c_float), ("greedy", C.c_int32), ("eos_id", C.c_int32),
                ("seed", C.c_uint64), ("top_k", C.c_int32), ("reserved", C.c_int32)]


class sd_round_out(C.Structure):
    _fields_ = [("K", C.c_int32), ("n_accepted", C.c_int32), ("n_new", C.c_int32),
                ("tokens", C.c_int32 * (SD_MAX_K + 1)), ("cand", C.c_int32 * SD_MAX_K), ("p_hat", C.c_float)]


class sd_stats(C.Structure):
    _fields_ = [("N", C.c_int64), ("N_draft", C.c_int64), ("N_target", C.c_int64), ("N_discarded", C.c_int64),
                ("rounds", C.c_int64), ("t_draft_s", C.c_double), ("t_target_s", C.c_double),
                ("t_accept_s", C.c_double), ("t_total_s", C.c_double)]


_i32p, _f32p, _u8p = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint8)
_PROTOS = {
    "sd_create": (C.c_int32, [C.POINTER(C.c_void_p), C.POINTER(sd_model), C.POINTER(sd_model), C.POINTER(sd_head),
                              C.POINTER(sd_config)]),
    "sd_destroy": (C.c_int32, [C.c_void_p]),
    "sd_prefill": (C.c_int32, [C.c_void_p, C.c_int32, _i32p, C.c_int32]),
    "specdec_round": (C.c_int32, [C.c_void_p, C.POINTER(sd_params), C.POINTER(sd_round_out)]),
    "specdec_generate": (C.c_int32, [C.c_void_p, C.POINTER(sd_params), C.c_int32, _i32p, _i32p, C.POINTER(sd_stats)]),
    "sd_accept_resample": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                       C.c_int32, C.POINTER(sd_params), C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]),
    "sd_accept_workspace_bytes": (C.c_int64, [C.c_int32, C.c_int32]),
    "sd_accept_resample_static": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                              C.c_int32, C.POINTER(sd_params), C.c_int32, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "sd_forward": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p, C.c_int32, _f32p, _f32p]),
    "sd_seq_state": (C.c_int32, [C.c_void_p, C.c_int32, _i32p, _i32p, _i32p, _i32p]),
    "sd_last_round_times": (C.c_int32, [C.c_void_p, C.POINTER(C.c_double), _i32p]),
    "sd_last_round_rows": (C.c_int32, [C.c_void_p, C.c_int32, _f32p, _f32p, _f32p]),
    "sd_profile_enable": (C.c_int32, [C.c_void_p, C.c_int32]),
    "sd_profile_read": (C.c_int32, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "sd_gemm_skinny": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p]),
    "sd_head_examples": (C.c_int32, [C.c_void_p, C.c_int32, _i32p, C.c_int32, C.c_int32, C.c_float, C.c_uint64, C.c_int32,
                                     C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, _i32p, _i32p]),
    "sd_trainer_create": (C.c_int32, [C.POINTER(C.c_void_p), C.POINTER(sd_head), C.c_int32, C.c_void_p]),
    "sd_trainer_destroy": (C.c_int32, [C.c_void_p]),
    "sd_trainer_step": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_float,
                                    C.c_float, C.c_float, C.c_float, C.c_float, C.c_int32, _f32p]),
    "sd_trainer_predict": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]),
    "sd_trainer_read": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, _f32p]),
    "sd_trainer_export": (C.c_int32, [C.c_void_p, C.c_int32, _vpp, _vpp]),
    "sd_mlp_act": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                               C.c_void_p, C.c_int32, C.c_void_p]),
    "sd_mlp_act_is_fused": (C.c_int32, [C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "sd_qkv_rope_is_fused": (C.c_int32, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "sd_qkv_rope": (C.c_int32, [C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]),
    "sd_gemm_tile": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.c_void_p]),
    "sd_gemm_tile_workspace_bytes": (C.c_int64, [C.c_int32, C.c_int32, C.c_int32]),
    "sd_gemm_workspace_bytes": (C.c_int64, [C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
    "sd_strerror": (C.c_char_p, [C.c_int32]),
    "sd_version": (C.c_char_p, []),
}
for _name, (_res, _args) in _PROTOS.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args

EXPORTS = sorted(_PROTOS)


class SpecDecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.sd_strerror(status).decode()} ({status})")


def _check(status: int, where: str) -> None:
    if status != SD_OK:
        raise SpecDecError(status, where)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SD_F32
    if dt == torch.bfloat16:
        return SD_BF16
    raise ValueError(f"unsupported dtype {dt}")


def _ptr_array(tensors: Sequence[torch.Tensor]):
    arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return arr


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_params(h: float = 0.7, temperature: float = 1.0, greedy: bool = False, eos_id: int = -1,
                seed: int = 0, top_k: int = 0) -> sd_params:
    return sd_params(float(h), float(temperature), int(bool(greedy)), int(eos_id), int(seed), int(top_k), 0)


def _model_struct(m: Dict, keep: list) -> sd_model:
    s = m["shape"]
    for t in [m["tok_emb"], m["lm_head"], m["final_norm"]] + [l[k] for l in m["layers"] for k in l]:
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("model tensors must be contiguous CUDA tensors")
    arrs = {k: _ptr_array([l[k] for l in m["layers"]])
            for k in ("wqkv", "wo", "w_gate_up", "w_down", "norm_attn", "norm_mlp")}
    keep.append(arrs)
    return sd_model(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                    _dtype_code(m["dtype"]), s.rope_theta, s.rms_eps, m["tok_emb"].data_ptr(),
                    m["lm_head"].data_ptr(), m["final_norm"].data_ptr(),
                    C.cast(arrs["wqkv"], _vpp), C.cast(arrs["wo"], _vpp), C.cast(arrs["w_gate_up"], _vpp),
                    C.cast(arrs["w_down"], _vpp), C.cast(arrs["norm_attn"], _vpp), C.cast(arrs["norm_mlp"], _vpp))


class Context:
    """Owns an sd_ctx.  `target`, `draft` and `head` are the dicts of
    `synth.make_model` / `synth.make_head` with CUDA tensors; they are kept alive here."""

    def __init__(self, target: Dict, draft: Dict, head: Optional[Dict], batch: int, max_seq: int, k_max: int):
        self._keep = [target, draft, head]
        tm, dm = _model_struct(target, self._keep), _model_struct(draft, self._keep)
        hp = None
        if head is not None:
            dims = (C.c_int32 * len(head["dims"]))(*head["dims"])
            W, b = _ptr_array(head["W"]), _ptr_array(head["b"])
            self._keep += [dims, W, b]
            hs = sd_head(len(head["W"]), C.cast(dims, _i32p), int(head["residual"]), _dtype_code(head["dtype"]),
                         C.cast(W, _vpp), C.cast(b, _vpp))
            hp = C.byref(hs)
        cfg = sd_config(batch, max_seq, k_max, _stream_ptr())
        self.handle = C.c_void_p()
        self.batch, self.max_seq, self.k_max = batch, max_seq, k_max
        self.vocab = target["shape"].vocab
        self.d_model = (target["shape"].d_model, draft["shape"].d_model)
        _check(lib.sd_create(C.byref(self.handle), C.byref(tm), C.byref(dm), hp, C.byref(cfg)), "sd_create")

    def close(self) -> None:
        if self.handle:
            lib.sd_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- entry points, named as in the header
    def sd_prefill(self, seq: int, prompt: Sequence[int]) -> None:
        arr = (C.c_int32 * len(prompt))(*prompt)
        _check(lib.sd_prefill(self.handle, seq, arr, len(prompt)), "sd_prefill")

    def specdec_round(self, params: sd_params) -> List[dict]:
        out = (sd_round_out * self.batch)()
        _check(lib.specdec_round(self.handle, C.byref(params), out), "specdec_round")
        return [dict(K=o.K, n=o.n_accepted, tokens=list(o.tokens[: o.n_new]), cand=list(o.cand[: o.K]),
                     p_hat=o.p_hat) for o in out]

    def specdec_generate(self, params: sd_params, max_new_tokens: int):
        toks = (C.c_int32 * (self.batch * max_new_tokens))()
        lens = (C.c_int32 * self.batch)()
        st = sd_stats()
        _check(lib.specdec_generate(self.handle, C.byref(params), max_new_tokens, toks, lens, C.byref(st)),
               "specdec_generate")
        seqs = [list(toks[b * max_new_tokens: b * max_new_tokens + lens[b]]) for b in range(self.batch)]
        stats = {k: getattr(st, k) for k, _ in sd_stats._fields_}
        return seqs, stats

    def sd_forward(self, which: int, seq: int, start: int, tokens: Sequence[int], want_hidden: bool = False):
        n = len(tokens)
        arr = (C.c_int32 * n)(*tokens)
        logits = torch.empty((n, self.vocab), dtype=torch.float32)
        hidden = torch.empty((n, self.d_model[which]), dtype=torch.float32) if want_hidden else None
        _check(lib.sd_forward(self.handle, which, seq, start, arr, n, C.cast(logits.data_ptr(), _f32p),
                              C.cast(hidden.data_ptr(), _f32p) if want_hidden else None), "sd_forward")
        return (logits, hidden) if want_hidden else logits

    def sd_seq_state(self, seq: int) -> dict:
        v = [C.c_int32() for _ in range(4)]
        _check(lib.sd_seq_state(self.handle, seq, *[C.byref(x) for x in v]), "sd_seq_state")
        return dict(P=v[0].value, kv_len_target=v[1].value, kv_len_draft=v[2].value, round=v[3].value)

    def sd_last_round_times(self) -> dict:
        t = (C.c_double * 3)()
        rows = C.c_int32()
        _check(lib.sd_last_round_times(self.handle, t, C.byref(rows)), "sd_last_round_times")
        return dict(t_draft_s=t[0], t_target_s=t[1], t_accept_s=t[2], target_rows=rows.value)

    def sd_last_round_rows(self, seq: int, K: int):
        q = torch.empty((K, self.vocab), dtype=torch.float32)
        p = torch.empty((K + 1, self.vocab), dtype=torch.float32)
        s = torch.zeros((max(K - 1, 1),), dtype=torch.float32)
        _check(lib.sd_last_round_rows(self.handle, seq, C.cast(q.data_ptr(), _f32p), C.cast(p.data_ptr(), _f32p),
                                      C.cast(s.data_ptr(), _f32p)), "sd_last_round_rows")
        return q, p, s[: K - 1]

    def sd_head_examples(self, seq: int, prompt: Sequence[int], response: Sequence[int], r: float, seed: int,
                         example: int, temperature: float = 1.0, top_k: int = 0):
        """(E [N, d] fp32, P [N] fp32, mask [N] int32) on the device, and Y, Z as lists."""
        toks = list(prompt) + list(response)
        N = len(response)
        arr = (C.c_int32 * len(toks))(*toks)
        dev = torch.device("cuda", torch.cuda.current_device())
        E = torch.empty((N, self.d_model[1]), dtype=torch.float32, device=dev)
        P = torch.empty((N,), dtype=torch.float32, device=dev)
        mask = torch.empty((N,), dtype=torch.int32, device=dev)
        Y, Z = (C.c_int32 * N)(), (C.c_int32 * N)()
        _check(lib.sd_head_examples(self.handle, seq, arr, len(prompt), N, r, seed, example, temperature, top_k,
                                    E.data_ptr(), P.data_ptr(), mask.data_ptr(), Y, Z), "sd_head_examples")
        return E, P, mask, list(Y), list(Z)

    def sd_profile_enable(self, every: int) -> None:
        _check(lib.sd_profile_enable(self.handle, every), "sd_profile_enable")

    def sd_profile_read(self) -> dict:
        n = (C.c_int64 * 5)()
        s = (C.c_double * 5)()
        b = (C.c_double * 5)()
        _check(lib.sd_profile_read(self.handle, n, s, b), "sd_profile_read")
        kinds = ("qkv", "o", "gate_up", "down", "lm_head")
        return {k: dict(launches=n[i], seconds=s[i], weight_bytes=b[i]) for i, k in enumerate(kinds)}


def sd_accept_resample(p_logits: torch.Tensor, q_logits: torch.Tensor, cand: torch.Tensor, K_per_seq: torch.Tensor,
                       params: sd_params, round_idx: int, out=None):
    """p_logits [B, Kmax+1, V] fp32, q_logits [B, Kmax, V] fp32, cand [B, Kmax] int32,
    K_per_seq [B] int32, all CUDA.  Returns (n [B], token [B], flags [B, Kmax]) CUDA tensors;
    enqueued on the current stream, not synchronised.  `out` may carry preallocated
    (n, token, flags, workspace) tensors; the call's status word (see the header) is
    workspace[B * (2 * Kmax + 1) * 16:][:4] as int32."""
    B, Kp1, V = p_logits.shape
    Kmax = Kp1 - 1
    assert q_logits.shape == (B, Kmax, V) and cand.shape == (B, Kmax) and K_per_seq.shape == (B,)
    for t, dt in ((p_logits, torch.float32), (q_logits, torch.float32), (cand, torch.int32), (K_per_seq, torch.int32)):
        assert t.is_cuda and t.is_contiguous() and t.dtype == dt
    if out is None:
        dev = p_logits.device
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Kmax), dtype=torch.uint8, device=dev),
               torch.empty(lib.sd_accept_workspace_bytes(B, Kmax), dtype=torch.uint8, device=dev))
    n, tok, flags, ws = out
    _check(lib.sd_accept_resample(p_logits.data_ptr(), q_logits.data_ptr(), cand.data_ptr(), K_per_seq.data_ptr(),
                                  B, Kmax, V, C.byref(params), round_idx, ws.data_ptr(), _stream_ptr(),
                                  n.data_ptr(), tok.data_ptr(), flags.data_ptr()), "sd_accept_resample")
    return n, tok, flags


def lib_static_max_batch() -> int:
    """SD_ACCEPT_STATIC_MAX_BATCH of the header."""
    return 64


def sd_accept_resample_static(p_logits: torch.Tensor, q_logits: torch.Tensor, cand: torch.Tensor,
                              K_per_seq: torch.Tensor, params: sd_params, round_idx: int, out):
    """sd_accept_resample with the library's static scratch: `out` = preallocated (n [B] int32,
    token [B] int32, flags [B, Kmax] uint8) CUDA tensors (this wrapper allocates nothing on the
    device either).  Returns the device address of the call's status word."""
    B, Kp1, V = p_logits.shape
    Kmax = Kp1 - 1
    assert q_logits.shape == (B, Kmax, V) and cand.shape == (B, Kmax) and K_per_seq.shape == (B,)
    for t, dt in ((p_logits, torch.float32), (q_logits, torch.float32), (cand, torch.int32), (K_per_seq, torch.int32)):
        assert t.is_cuda and t.is_contiguous() and t.dtype == dt
    n, tok, flags = out
    assert n.shape == (B,) and tok.shape == (B,) and flags.shape == (B, Kmax)
    word = C.c_void_p()
    _check(lib.sd_accept_resample_static(p_logits.data_ptr(), q_logits.data_ptr(), cand.data_ptr(),
                                         K_per_seq.data_ptr(), B, Kmax, V, C.byref(params), round_idx, _stream_ptr(),
                                         n.data_ptr(), tok.data_ptr(), flags.data_ptr(), C.byref(word)),
           "sd_accept_resample_static")
    return word.value


def sd_gemm_skinny(W: torch.Tensor, X: torch.Tensor, out=None) -> torch.Tensor:
    """Y = X W^T in fp32.  W [N, K], X [M, K], same dtype (fp32 or bf16), CUDA, contiguous."""
    assert W.is_cuda and X.is_cuda and W.is_contiguous() and X.is_contiguous() and W.dtype == X.dtype
    (N, K), (M, K2) = W.shape, X.shape
    assert K == K2
    dt = _dtype_code(W.dtype)
    if out is None:
        nbytes = lib.sd_gemm_workspace_bytes(dt, M, N, K)
        if nbytes <= 0:
            raise SpecDecError(SD_EINVAL, "sd_gemm_workspace_bytes")
        out = (torch.empty((M, N), dtype=torch.float32, device=W.device),
               torch.empty(nbytes, dtype=torch.uint8, device=W.device))
    Y, ws = out
    _check(lib.sd_gemm_skinny(dt, W.data_ptr(), X.data_ptr(), M, N, K, Y.data_ptr(), ws.data_ptr(), _stream_ptr()),
           "sd_gemm_skinny")
    return Y


def sd_mlp_act(W_gate_up: torch.Tensor, X: torch.Tensor, mode: int = -1) -> torch.Tensor:
    """silu(X Wg^T) * (X Wu^T) in the inputs' dtype.  W_gate_up [2 ffn, K] = [gate; up], X [M, K], CUDA, contiguous.
    mode 1: the one-launch kernel, 0: product + activation kernel, -1: the forward passes' choice."""
    W = W_gate_up
    assert W.is_cuda and X.is_cuda and W.is_contiguous() and X.is_contiguous() and W.dtype == X.dtype
    (N2, K), (M, K2) = W.shape, X.shape
    assert K == K2 and N2 % 2 == 0
    dt = _dtype_code(W.dtype)
    act = torch.empty((M, N2 // 2), dtype=W.dtype, device=W.device)
    nbytes = lib.sd_gemm_workspace_bytes(dt, M, N2, K)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    _check(lib.sd_mlp_act(dt, W.data_ptr(), X.data_ptr(), M, N2 // 2, K, act.data_ptr(), ws.data_ptr(), mode,
                          _stream_ptr()), "sd_mlp_act")
    return act


def sd_mlp_act_is_fused(dtype: torch.dtype, M: int, ffn: int, K: int) -> bool:
    return bool(lib.sd_mlp_act_is_fused(_dtype_code(dtype), M, ffn, K))


def sd_qkv_rope(W_qkv: torch.Tensor, X: torch.Tensor, n_heads: int, n_kv_heads: int, head_dim: int,
                row_seq: torch.Tensor, row_pos: torch.Tensor, cos_sin: torch.Tensor, q_out: torch.Tensor,
                k_cache: torch.Tensor, v_cache: torch.Tensor, mode: int = -1) -> None:
    """q|k|v product of a decoder layer, rotary embedding, q -> q_out [M, Hq hd], k -> k_cache [n_seq, Hkv, max_seq, hd],
    v -> v_cache [n_seq, Hkv, hd, max_seq] at (row_seq[m], row_pos[m]); rows with row_seq < 0 write nothing.
    cos_sin: fp32 [max_seq, hd / 2, 2].  mode 1: one launch, 0: product + rotary kernel, -1: the forward passes' choice."""
    W = W_qkv
    for t in (W, X, row_seq, row_pos, cos_sin, q_out, k_cache, v_cache):
        assert t.is_cuda and t.is_contiguous()
    (N, K), (M, K2) = W.shape, X.shape
    max_seq = k_cache.shape[2]
    assert K == K2 and N == (n_heads + 2 * n_kv_heads) * head_dim and W.dtype == X.dtype == q_out.dtype
    assert k_cache.dtype == W.dtype and v_cache.dtype == W.dtype
    assert row_seq.dtype == torch.int32 and row_pos.dtype == torch.int32 and row_seq.numel() == M == row_pos.numel()
    assert cos_sin.dtype == torch.float32 and tuple(cos_sin.shape) == (max_seq, head_dim // 2, 2)
    assert tuple(q_out.shape) == (M, n_heads * head_dim)
    assert tuple(k_cache.shape[1:]) == (n_kv_heads, max_seq, head_dim)
    assert tuple(v_cache.shape) == (k_cache.shape[0], n_kv_heads, head_dim, max_seq)
    dt = _dtype_code(W.dtype)
    nbytes = lib.sd_gemm_workspace_bytes(dt, M, N, K)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    _check(lib.sd_qkv_rope(dt, W.data_ptr(), X.data_ptr(), M, n_heads, n_kv_heads, head_dim, K, row_seq.data_ptr(),
                           row_pos.data_ptr(), cos_sin.data_ptr(), q_out.data_ptr(), k_cache.data_ptr(),
                           v_cache.data_ptr(), max_seq, ws.data_ptr(), mode, _stream_ptr()), "sd_qkv_rope")


def sd_qkv_rope_is_fused(dtype: torch.dtype, M: int, n_heads: int, n_kv_heads: int, head_dim: int, K: int) -> bool:
    return bool(lib.sd_qkv_rope_is_fused(_dtype_code(dtype), M, n_heads, n_kv_heads, head_dim, K))


def sd_gemm_tile(W: torch.Tensor, X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y = X W^T in fp32 through the large-M kernel.  W [N, K], X [M, K], bf16, CUDA, contiguous."""
    assert W.is_cuda and X.is_cuda and W.is_contiguous() and X.is_contiguous()
    assert W.dtype == torch.bfloat16 and X.dtype == torch.bfloat16
    (N, K), (M, K2) = W.shape, X.shape
    assert K == K2
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float32, device=W.device)
    nbytes = lib.sd_gemm_tile_workspace_bytes(M, N, K)
    if nbytes < 0:
        raise SpecDecError(SD_EINVAL, "sd_gemm_tile_workspace_bytes")
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    _check(lib.sd_gemm_tile(W.data_ptr(), X.data_ptr(), M, N, K, Y.data_ptr(), ws.data_ptr(), _stream_ptr()),
           "sd_gemm_tile")
    return Y


def _head_struct(head: Dict, keep: list) -> sd_head:
    dims = (C.c_int32 * len(head["dims"]))(*head["dims"])
    W, b = _ptr_array(head["W"]), _ptr_array(head["b"])
    keep += [dims, W, b]
    return sd_head(len(head["W"]), C.cast(dims, _i32p), int(head["residual"]), _dtype_code(head["dtype"]),
                   C.cast(W, _vpp), C.cast(b, _vpp))


class Trainer:
    """Owns an sd_trainer initialised from a head dict of `synth.make_head` (CUDA tensors)."""

    def __init__(self, head: Dict, n_max: int):
        self._keep = [head]
        hs = _head_struct(head, self._keep)
        self.handle = C.c_void_p()
        self.dims, self.residual = list(head["dims"]), bool(head["residual"])
        _check(lib.sd_trainer_create(C.byref(self.handle), C.byref(hs), n_max, _stream_ptr()), "sd_trainer_create")

    def close(self):
        if self.handle:
            lib.sd_trainer_destroy(self.handle)
            self.handle = C.c_void_p()

    def sd_trainer_step(self, E: torch.Tensor, P: torch.Tensor, mask: torch.Tensor, w_acc=1.0, w_rej=1.0, lr=5e-5,
                        beta1=0.9, beta2=0.999, eps=1e-8, apply=True, want_loss=True) -> Optional[float]:
        assert E.is_cuda and E.dtype == torch.float32 and E.is_contiguous() and E.shape[1] == self.dims[0]
        assert P.is_cuda and P.dtype == torch.float32 and mask.is_cuda and mask.dtype == torch.int32
        n = E.shape[0]
        assert P.numel() == n and mask.numel() == n
        loss = C.c_float()
        _check(lib.sd_trainer_step(self.handle, E.data_ptr(), P.data_ptr(), mask.data_ptr(), n, w_acc, w_rej, lr, beta1,
                                   beta2, eps, int(bool(apply)), C.byref(loss) if want_loss else None),
               "sd_trainer_step")
        return loss.value if want_loss else None

    def sd_trainer_predict(self, E: torch.Tensor) -> torch.Tensor:
        out = torch.empty(E.shape[0], dtype=torch.float32, device=E.device)
        _check(lib.sd_trainer_predict(self.handle, E.data_ptr(), E.shape[0], out.data_ptr()), "sd_trainer_predict")
        return out

    def sd_trainer_read(self, layer: int, what: int) -> torch.Tensor:
        shape = (self.dims[layer + 1], self.dims[layer]) if what in (0, 2) else (self.dims[layer + 1],)
        out = torch.empty(shape, dtype=torch.float32)
        _check(lib.sd_trainer_read(self.handle, layer, what, C.cast(out.data_ptr(), _f32p)), "sd_trainer_read")
        return out

    def sd_trainer_export(self, dtype: torch.dtype, device="cuda") -> Dict:
        """A head dict (like synth.make_head's) holding the current weights in `dtype`."""
        L = len(self.dims) - 1
        W = [torch.empty((self.dims[j + 1], self.dims[j]), dtype=dtype, device=device) for j in range(L)]
        b = [torch.empty((self.dims[j + 1],), dtype=dtype, device=device) for j in range(L)]
        Wp, bp = _ptr_array(W), _ptr_array(b)
        _check(lib.sd_trainer_export(self.handle, _dtype_code(dtype), C.cast(Wp, _vpp), C.cast(bp, _vpp)),
               "sd_trainer_export")
        return dict(dims=list(self.dims), W=W, b=b, residual=self.residual, dtype=dtype)
