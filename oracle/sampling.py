"""Softmax, one-uniform sampling, and the accept / residual-resample step
(Appendix C rejection sampling; Algorithm 1's tail, shared by Algorithm 2).

Test infrastructure only (see oracle/__init__.py).

Readings where the paper is silent:
  * a sample from weights f with one uniform u is the inverse CDF in index
    order: y = min{v : c_v > u*S}, c_v = f_0 + ... + f_v summed left to right,
    S = c_{V-1}; if rounding leaves no such v, the largest v with f_v > 0;
  * the accept test for r in [0,1) is  r < p(y)/q(y), evaluated without the
    division as r*q(y) < p(y);
  * a residual whose mass is numerically zero falls back to p_{n+1};
  * greedy mode compares y_i with argmax p_i (Sec. 4.1), ties to the lowest id;
  * top-k warping (Appendix D.1) keeps every logit >= the k-th largest of its row.

Pins: chi-square of the emitted token against p on tiny vocabularies, the
acceptance frequency sum_v min(p_v, q_v), p == q accepts everything, and the
constant-alpha closed form (1 - alpha^(K+1)) / (1 - alpha).
"""
from __future__ import annotations

import numpy as np

from . import philox


def softmax(logits: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - np.max(z, axis=-1, keepdims=True)
    ez = np.exp(z)
    return ez / np.sum(ez, axis=-1, keepdims=True)


def warp_top_k(logits: np.ndarray, top_k: int) -> np.ndarray:
    """Top-k warping of the paper's inference setting (Appendix D.1, k = 50): logits
    below the k-th largest value of their row become -inf, so the softmax that follows
    gives them probability 0.  Entries equal to the k-th largest value are all kept.
    top_k <= 0 or >= V leaves the row unchanged."""
    z = np.asarray(logits, dtype=np.float64)
    v = z.shape[-1]
    if top_k <= 0 or top_k >= v:
        return z
    kth = np.partition(z, v - top_k, axis=-1)[..., v - top_k]
    return np.where(z >= kth[..., None], z, -np.inf)


def argmax_lowest(x: np.ndarray) -> int:
    """Index of the maximum; the lowest index among ties."""
    return int(np.argmax(np.asarray(x)))      # numpy returns the first maximum


def sample_inverse_cdf(f: np.ndarray, u: float) -> int:
    """Draw from non-negative weights f (need not be normalised) with one uniform."""
    f = np.asarray(f, dtype=np.float64)
    c = np.cumsum(f)                           # sequential left-to-right sum
    thresh = u * c[-1]
    hit = np.nonzero(c > thresh)[0]
    if hit.size:
        return int(hit[0])
    pos = np.nonzero(f > 0)[0]
    return int(pos[-1])


def residual(p: np.ndarray, q: np.ndarray) -> np.ndarray:
    """(p - q)_+ , unnormalised."""
    return np.maximum(np.asarray(p, dtype=np.float64) - np.asarray(q, dtype=np.float64), 0.0)


def cdf_margin(f: np.ndarray, u: float, y: int) -> float:
    """Distance, as a fraction of the total mass, from u*S to the nearer edge of
    token y's bucket [c_{y-1}, c_y): how close the draw was to picking a neighbour."""
    f = np.asarray(f, dtype=np.float64)
    c = np.cumsum(f)
    lo = c[y - 1] if y > 0 else 0.0
    return float(min(abs(c[y] - u * c[-1]), abs(u * c[-1] - lo)) / c[-1])


def top2_gap(x: np.ndarray) -> float:
    """(largest - second largest) / max|x|: the margin of an argmax decision."""
    x = np.asarray(x, dtype=np.float64)
    top = np.partition(x, -2)[-2:]
    return float((top[1] - top[0]) / max(np.max(np.abs(x)), 1e-300))


def accept_resample(p_logits, q_logits, cand, K: int, *, temperature: float = 1.0,
                    greedy: bool = False, seed: int = 0, rnd: int = 0, seq: int = 0,
                    forced: dict | None = None, top_k: int = 0) -> dict:
    """Verify K candidates and produce the correction / bonus token.

    p_logits: [>=K+1, V] target logits for positions 1..K+1; q_logits: [>=K, V]
    draft logits for positions 1..K; cand: the K candidates y_1..y_K.

    Returns dict(n, token, flags[K], ratio[K], r[K], u, margin) where flags[i-1]
    is the outcome of the i-th accept test taken on its own, n is the index of the
    first failed test (K if none), token is y', and margin is the decision margin
    of y' (bucket-edge distance, or top-2 gap in greedy mode).

    `forced` lets a parity harness push the oracle through a near-tie the other
    way: {("accept", i): 0/1} replaces the i-th test's outcome and {"token": t}
    replaces y'.  Nothing else uses it.
    """
    forced = forced or {}
    p_logits = np.asarray(p_logits, dtype=np.float64)
    q_logits = np.asarray(q_logits, dtype=np.float64)
    cand = [int(c) for c in np.asarray(cand).reshape(-1)[:K]]
    flags = np.zeros(K, dtype=np.uint8)
    ratio = np.zeros(K, dtype=np.float64)
    rs = np.zeros(K, dtype=np.float64)

    if greedy:
        for i in range(1, K + 1):
            flags[i - 1] = 1 if cand[i - 1] == argmax_lowest(p_logits[i - 1]) else 0
            ratio[i - 1] = top2_gap(p_logits[i - 1])
            if ("accept", i) in forced:
                flags[i - 1] = forced[("accept", i)]
        n = int(np.argmin(flags)) if not flags.all() else K
        token = forced.get("token", argmax_lowest(p_logits[n]))
        return dict(n=n, token=int(token), flags=flags, ratio=ratio, r=rs, u=None,
                    margin=top2_gap(p_logits[n]))

    # both models are warped the same way before the softmax (Appendix D.1)
    p = softmax(warp_top_k(p_logits[:K + 1], top_k), temperature)
    q = softmax(warp_top_k(q_logits[:K], top_k), temperature) if K > 0 else np.zeros((0, p.shape[1]))
    for i in range(1, K + 1):
        y = cand[i - 1]
        r = philox.uniform(seed, i, rnd, seq, philox.STREAM_ACCEPT)
        rs[i - 1] = r
        ratio[i - 1] = p[i - 1, y] / q[i - 1, y] if q[i - 1, y] > 0 else np.inf
        flags[i - 1] = 1 if r * q[i - 1, y] < p[i - 1, y] else 0
        if ("accept", i) in forced:
            flags[i - 1] = forced[("accept", i)]
    n = K
    for i in range(1, K + 1):
        if not flags[i - 1]:
            n = i - 1
            break
    u = philox.uniform(seed, n + 1, rnd, seq, philox.STREAM_RESAMPLE)
    if n < K:
        f = residual(p[n], q[n])
        if not (f.sum() > 0.0):
            f = p[n]
    else:
        f = p[K]
    token = sample_inverse_cdf(f, u)
    margin = cdf_margin(f, u, token)
    token = int(forced.get("token", token))
    return dict(n=n, token=token, flags=flags, ratio=ratio, r=rs, u=u, margin=margin)
