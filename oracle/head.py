"""Acceptance-prediction head (Eq. 3) and the threshold stop rule (Sec. 4.3).

Test infrastructure only (see oracle/__init__.py).

Sec. 5.1 describes the head only as a "(D+1)-layer ResNet with SiLU".  Reading
taken: D hidden layers z <- SiLU(W_j z + b_j), with the skip connection
z <- z + SiLU(W_j z + b_j) when `residual` is set and the layer is square; the
last layer is linear to one logit; Eq. (3) applies the sigmoid.

Stop rule: the predicted probability that at least one of the first k
candidates is rejected is 1 - prod_{i<=k} P_hat_i (chain rule, Sec. 4.3); the
round stops when it is strictly greater than h.

Pins: brute-force search of the stop index on small inputs; closed-form special
cases (h >= 1, h < 0, constant s); a D = 0 head equals a logistic regression.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass
class HeadWeights:
    W: List[np.ndarray]      # W[j]: [dims[j+1], dims[j]]; last one has a single row
    b: List[np.ndarray]      # b[j]: [dims[j+1]]
    residual: bool = False


def sigmoid(z: float) -> float:
    z = float(z)
    if z >= 0:
        return 1.0 / (1.0 + np.exp(-z))
    ez = np.exp(z)
    return float(ez / (1.0 + ez))


def head_logit(head: HeadWeights, e: np.ndarray) -> float:
    """f_theta(e): the pre-sigmoid scalar."""
    z = np.asarray(e, dtype=np.float64)
    n = len(head.W)
    for j in range(n - 1):
        W = np.asarray(head.W[j], dtype=np.float64)
        a = W @ z + np.asarray(head.b[j], dtype=np.float64)
        a = a / (1.0 + np.exp(-a))                       # SiLU
        z = z + a if (head.residual and W.shape[0] == W.shape[1]) else a
    W = np.asarray(head.W[n - 1], dtype=np.float64)
    return float((W @ z + np.asarray(head.b[n - 1], dtype=np.float64))[0])


def accept_prob(head: HeadWeights, e: np.ndarray) -> float:
    """Eq. (3): predicted conditional acceptance probability of the token whose
    final embedding is e."""
    return sigmoid(head_logit(head, e))


def should_stop(p_hat: float, h: float) -> bool:
    """Stop iff the predicted probability of at least one rejection, 1 - p_hat,
    exceeds h (strictly)."""
    return (1.0 - p_hat) > h


def candidate_length(s, h: float, k_cap: int) -> int:
    """Candidate length K of a round of Algorithm 2 when the head's outputs would
    be s[0], s[1], ... for y_1, y_2, ... and no manual stop fires before k_cap.

    The prediction for y_{i-1} becomes available in the forward that yields q_i,
    so y_i is drawn before the test that uses s_1..s_{i-1}; nothing is multiplied
    in at i = 1 (there is no e_0).
    """
    p_hat = 1.0
    for i in range(1, k_cap + 1):
        if i > 1:
            p_hat *= float(s[i - 2])
        if should_stop(p_hat, h):
            return i
    return k_cap
