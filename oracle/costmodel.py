"""Inference-time decomposition of speculative decoding (Sec. 3.2, Sec. 5.1).

Test infrastructure only (see oracle/__init__.py).

Eq. (1):  T_total = t_draft * N_draft + t_target * N_target
Lemma 1 / Eq. (2):  T_total = t_draft * N + t_draft * N_discarded + (t_target - t_draft) * N_target,
          which follows from N_draft + N_target = N + N_discarded
Eq. (4):  latency per token = t_draft + t_draft * (N_discarded / N) + (t_target - t_draft) * (N_target / N)

Pins: the paper's printed numbers (tests/golden/paper_throughput.txt): the
stand-alone target time gives its tokens/s, and the printed tokens/s divide to
the printed speed-ups.
"""
from __future__ import annotations


def total_time(t_draft: float, t_target: float, n_draft: int, n_target: int) -> float:
    """Eq. (1)."""
    return t_draft * n_draft + t_target * n_target


def total_time_decomposed(t_draft: float, t_target: float, n: int, n_discarded: int, n_target: int) -> float:
    """Lemma 1 / Eq. (2)."""
    return t_draft * n + t_draft * n_discarded + (t_target - t_draft) * n_target


def latency_per_token(t_draft: float, t_target: float, discard_rate: float, verification_rate: float) -> float:
    """Eq. (4): discard_rate = N_discarded / N, verification_rate = N_target / N."""
    return t_draft + t_draft * discard_rate + (t_target - t_draft) * verification_rate


def tokens_per_second(t_draft: float, t_target: float, discard_rate: float, verification_rate: float) -> float:
    return 1.0 / latency_per_token(t_draft, t_target, discard_rate, verification_rate)


def target_only_tokens_per_second(t_target_standalone: float) -> float:
    """Plain autoregressive decoding: one target forward per token."""
    return 1.0 / t_target_standalone
