"""Training of the acceptance-prediction head (Sec. 4.4): training-set construction
with token mixing, the weighted binary cross-entropy, its gradient through the
head of Eq. (3), and Adam.

Test infrastructure only (see oracle/__init__.py).

Steps, in the paper's order and notation, for one prompt and one target response
X_1..X_N (positions are 1-based in the response):

  q_i = q(. | prompt, X_<i),  p_i = p(. | prompt, X_<i)          one forward of each model
  Y_i ~ q_i                                                       u(slot i, example, stream 3)
  P_i = min(1, p_i(Y_i) / q_i(Y_i))                               the training target
  Z_i = X_i with probability r, else Y_i                          u(slot i, example, stream 4) < r
  E_i = draft's final embedding of Z_i given (prompt, Z_<i)       second draft forward
  P_hat_i = sigmoid(f_theta(E_i))
  loss = (1/n) sum over {i : Z_i = Y_i} of
         - w_acc P_i log P_hat_i - w_rej (1 - P_i) log(1 - P_hat_i)

Readings where the paper is silent: the paper writes the loss as a plain sum; here it
is divided by the number n of tokens that carry a loss (this only rescales the learning
rate).  "final embedding" is the draft's hidden state after its last RMSNorm, the same
vector the round feeds the head.  The optimiser is Adam (Kingma & Ba) with bias
correction and no weight decay (Appendix D.1 names Adam only).  Top-k warping and
the temperature apply to p_i and q_i as in the round.

Pins: the gradient against central finite differences and against torch autograd
on binary_cross_entropy_with_logits; Adam against torch.optim.Adam; targets in
[0, 1] and equal to 1 when the two models coincide; the mixing fraction.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from . import philox
from .head import HeadWeights
from .model import ModelWeights, forward_full
from .sampling import sample_inverse_cdf, softmax, warp_top_k

STREAM_LABEL = 3
STREAM_MIX = 4


def labels(p_logits, q_logits, seed: int, example: int, seq: int = 0, temperature: float = 1.0, top_k: int = 0):
    """Y_i ~ q_i and P_i = min(1, p_i(Y_i)/q_i(Y_i)) for rows i = 1..N of the two
    logits arrays [N, V].  Returns (Y int array, P float array)."""
    p = softmax(warp_top_k(p_logits, top_k), temperature)
    q = softmax(warp_top_k(q_logits, top_k), temperature)
    n = p.shape[0]
    Y = np.zeros(n, dtype=np.int64)
    P = np.zeros(n, dtype=np.float64)
    for i in range(1, n + 1):
        u = philox.uniform(seed, i, example, seq, STREAM_LABEL)
        y = sample_inverse_cdf(q[i - 1], u)
        Y[i - 1] = y
        P[i - 1] = min(1.0, p[i - 1, y] / q[i - 1, y])
    return Y, P


def mix_tokens(X, Y, r: float, seed: int, example: int, seq: int = 0):
    """Token mixing: Z_i = X_i when u_i < r, else Y_i.  Returns (Z, mask) with
    mask_i = 1 where Z_i was taken from Y_i (the tokens that carry a loss)."""
    n = len(X)
    Z = np.zeros(n, dtype=np.int64)
    mask = np.zeros(n, dtype=np.int64)
    for i in range(1, n + 1):
        u = philox.uniform(seed, i, example, seq, STREAM_MIX)
        if u < r:
            Z[i - 1] = X[i - 1]
        else:
            Z[i - 1] = Y[i - 1]
            mask[i - 1] = 1
    return Z, mask


def make_examples(target: ModelWeights, draft: ModelWeights, prompt, X, r: float, seed: int, example: int,
                  temperature: float = 1.0, top_k: int = 0):
    """The training examples of one (prompt, response) pair: (E [N, d], P [N], mask [N],
    Y [N], Z [N])."""
    prompt = [int(t) for t in prompt]
    X = [int(t) for t in X]
    n0, N = len(prompt), len(X)
    p_logits, _ = forward_full(target, prompt + X)
    q_logits, _ = forward_full(draft, prompt + X)
    # the row of the token before X_i predicts position i
    Y, P = labels(p_logits[n0 - 1:n0 - 1 + N], q_logits[n0 - 1:n0 - 1 + N], seed, example, 0, temperature, top_k)
    Z, mask = mix_tokens(X, Y, r, seed, example)
    _, hid = forward_full(draft, prompt + [int(z) for z in Z])
    E = hid[n0:n0 + N]
    return E, P, mask, Y, Z


def _silu(a):
    return a / (1.0 + np.exp(-a))


def _silu_grad(a):
    s = 1.0 / (1.0 + np.exp(-a))
    return s * (1.0 + a * (1.0 - s))


def head_forward_batch(head: HeadWeights, E):
    """Logits f_theta(E_i) for a batch [n, d] plus what the backward pass needs."""
    z = np.asarray(E, dtype=np.float64)
    zs, pres = [z], []
    nl = len(head.W)
    for j in range(nl - 1):
        W = np.asarray(head.W[j], dtype=np.float64)
        a = z @ W.T + np.asarray(head.b[j], dtype=np.float64)
        pres.append(a)
        act = _silu(a)
        z = z + act if (head.residual and W.shape[0] == W.shape[1]) else act
        zs.append(z)
    W = np.asarray(head.W[nl - 1], dtype=np.float64)
    logit = (z @ W.T + np.asarray(head.b[nl - 1], dtype=np.float64))[:, 0]
    return logit, zs, pres


def weighted_bce(logit, P, mask, w_acc: float, w_rej: float):
    """(loss, d loss / d logit): the weighted BCE of Sec. 4.4 averaged over the masked
    tokens, written with log-sigmoid so that large |logit| stays finite."""
    logit = np.asarray(logit, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    m = np.asarray(mask, dtype=np.float64)
    n = max(m.sum(), 1.0)
    log_s = -np.logaddexp(0.0, -logit)          # log sigmoid(logit)
    log_1ms = -np.logaddexp(0.0, logit)         # log (1 - sigmoid(logit))
    s = np.exp(log_s)
    loss = np.sum(m * (-w_acc * P * log_s - w_rej * (1.0 - P) * log_1ms)) / n
    dlogit = m * (-w_acc * P * (1.0 - s) + w_rej * (1.0 - P) * s) / n
    return float(loss), dlogit


def head_loss_grad(head: HeadWeights, E, P, mask, w_acc: float = 1.0, w_rej: float = 1.0):
    """Loss and its gradient with respect to every W_j and b_j (lists like head.W / head.b)."""
    logit, zs, pres = head_forward_batch(head, E)
    loss, dlogit = weighted_bce(logit, P, mask, w_acc, w_rej)
    nl = len(head.W)
    gW: List[np.ndarray] = [None] * nl
    gb: List[np.ndarray] = [None] * nl
    dl = dlogit[:, None]                                      # [n, 1]
    gW[nl - 1] = dl.T @ zs[nl - 1]
    gb[nl - 1] = dl.sum(0)
    dz = dl @ np.asarray(head.W[nl - 1], dtype=np.float64)    # [n, d_last]
    for j in range(nl - 2, -1, -1):
        W = np.asarray(head.W[j], dtype=np.float64)
        skip = head.residual and W.shape[0] == W.shape[1]
        da = dz * _silu_grad(pres[j])
        gW[j] = da.T @ zs[j]
        gb[j] = da.sum(0)
        dz_in = da @ W
        dz = dz_in + dz if skip else dz_in
    return loss, gW, gb


@dataclass
class AdamState:
    m: List[np.ndarray] = field(default_factory=list)
    v: List[np.ndarray] = field(default_factory=list)
    t: int = 0


def adam_step(params: List[np.ndarray], grads: List[np.ndarray], state: AdamState, lr: float, beta1: float = 0.9,
              beta2: float = 0.999, eps: float = 1e-8) -> None:
    """One Adam update, in place, with bias correction."""
    if not state.m:
        state.m = [np.zeros_like(p, dtype=np.float64) for p in params]
        state.v = [np.zeros_like(p, dtype=np.float64) for p in params]
    state.t += 1
    c1 = 1.0 - beta1 ** state.t
    c2 = 1.0 - beta2 ** state.t
    for p, g, m, v in zip(params, grads, state.m, state.v):
        m *= beta1
        m += (1.0 - beta1) * g
        v *= beta2
        v += (1.0 - beta2) * g * g
        p -= lr * (m / c1) / (np.sqrt(v / c2) + eps)


def train_steps(head: HeadWeights, batches, w_acc: float, w_rej: float, lr: float, beta1: float = 0.9,
                beta2: float = 0.999, eps: float = 1e-8):
    """Runs Adam over `batches` (an iterable of (E, P, mask)); updates head in place
    (its arrays must be float64) and returns the per-step losses."""
    state = AdamState()
    losses = []
    for E, P, mask in batches:
        loss, gW, gb = head_loss_grad(head, E, P, mask, w_acc, w_rej)
        adam_step(head.W + head.b, gW + gb, state, lr, beta1, beta2, eps)
        losses.append(loss)
    return losses
