"""One SpecDec++ round (Algorithm 2), the generation loop around it with the
counters of Sec. 3.2, and the plain target-only definition of greedy decoding.

Test infrastructure only (see oracle/__init__.py).

Steps of a round, in the paper's order and notation (x = prefix, P = len(x),
rho = round index):

  p_hat <- 1
  for i = 1 .. K_cap:                                    K_cap = min(K_max, max_seq - P - 1)
      one draft forward over (x, y_1..y_{i-1}) gives the logits of q_i and, for
      i > 1, the final embedding e_{i-1} of y_{i-1}
      y_i ~ q_i  with u(rho, i, stream 0)               (argmax in greedy mode)
      if i > 1:  p_hat <- p_hat * sigmoid(f_theta(e_{i-1}))
      if 1 - p_hat > h:  break
      if y_i == EOS:     break                           (manual stop, Sec. 4.2 footnote)
  K <- number of candidates drawn
  p_1..p_{K+1} <- one target forward over (x, y_1..y_K), last K+1 rows
  r_i = u(rho, i, stream 1);  n = first i-1 with r_i >= p_i(y_i)/q_i(y_i), else K
  y' ~ Norm[(p_{n+1} - q_{n+1})_+]  if n < K  else  y' ~ p_{K+1}, with u(rho, n+1, stream 2)
  x <- x, y_1..y_n, y'

The loop bound is missing in the paper's listing; Sec. 5.1's manual cap on the
number of candidates is read as the bound K_max.  Nothing is multiplied into
p_hat at i = 1 because e_0 is never computed.

Pins: greedy generation equals target-only greedy decoding token for token
(Sec. 4.1); N_draft + N_target = N + N_discarded (Sec. 3.2); h >= 1 gives the
fixed-K algorithm; full-recompute and cached forwards give the same rounds; the
hindsight policy of Theorem 1 played through the rounds discards nothing and is
optimal among all stopping policies (brute force over every policy on tiny inputs).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np

from . import philox
from .head import HeadWeights, accept_prob, should_stop
from .model import CachedForward, ModelWeights, forward_full
from .sampling import (accept_resample, argmax_lowest, cdf_margin, sample_inverse_cdf, softmax,
                       top2_gap, warp_top_k)


@dataclass
class Params:
    h: float = 0.7
    temperature: float = 1.0
    greedy: bool = False
    eos_id: int = -1          # < 0: none
    seed: int = 0
    top_k: int = 0            # 0: full vocabulary; k > 0: top-k warping of both models (Appendix D.1)


@dataclass
class Stats:
    N: int = 0                # tokens kept in the output
    N_draft: int = 0          # draft forwards = candidates drawn
    N_target: int = 0         # target forwards = rounds
    N_discarded: int = 0      # candidates drawn and not accepted
    K_hist: List[int] = field(default_factory=list)
    n_hist: List[int] = field(default_factory=list)


class Recompute:
    """Forward by recomputing the whole prefix on every call (definitional mode)."""

    def __init__(self, w: ModelWeights):
        self.w = w

    def tail(self, tokens, m: int):
        """(logits, hidden) of the last m positions of `tokens`."""
        logits, hid = forward_full(self.w, tokens)
        return logits[-m:], hid[-m:]


class Cached:
    """Forward through `CachedForward`; re-uses whatever prefix of the cache
    matches the requested tokens and truncates the rest (the oracle's rollback)."""

    def __init__(self, w: ModelWeights):
        self.fw = CachedForward(w)
        self.toks: List[int] = []

    def tail(self, tokens, m: int):
        tokens = [int(t) for t in tokens]
        common = 0
        for a, b in zip(self.toks, tokens):
            if a != b:
                break
            common += 1
        keep = min(common, len(tokens) - m)
        self.fw.truncate(keep)
        logits, hid = self.fw.extend(tokens[keep:])
        self.toks = tokens
        return logits[-m:], hid[-m:]


def oracle_round(target, draft, head: Optional[HeadWeights], x: List[int], rho: int, params: Params,
                 k_max: int, max_seq: int, seq: int = 0, forced: Optional[dict] = None) -> dict:
    """One round on prefix x.  `target` / `draft` expose tail(tokens, m).

    Returns dict(K, n, cand, tokens (= y_1..y_n, y'), q_logits, p_logits, s (head
    outputs used), p_hat, trace) where trace lists every decision with its margin
    so a parity harness can tell a near-tie from an error.  `forced` maps
    ("draft", i) / ("stop", i) / ("accept", i) / "token" to a decision to impose;
    forced["K"] = k makes the round draw exactly k candidates whatever the stop rule
    says (0 <= k <= K_cap; k = 0 is a plain target step: Algorithm 1's tail with no
    candidate, y' ~ p_1), which is how a stopping policy other than the head's is
    played, e.g. the hindsight policy of Sec. 4.1.
    """
    forced = forced or {}
    P = len(x)
    k_cap = min(k_max, max_seq - P - 1)
    if k_cap < 1:
        raise OverflowError("sequence would overflow max_seq")
    trace = []
    cand: List[int] = []
    q_rows = []
    s_used = []
    p_hat = 1.0
    k_forced = forced.get("K")
    if k_forced is not None and not 0 <= k_forced <= k_cap:
        raise ValueError("forced K outside [0, K_cap]")
    for i in range(1, k_cap + 1):
        if k_forced is not None and i > k_forced:
            break
        logits, hid = draft.tail(x + cand, 1)
        q_rows.append(logits[0])
        if params.greedy:
            y = argmax_lowest(logits[0])
            trace.append(("draft", i, y, top2_gap(logits[0])))
        else:
            qi = softmax(warp_top_k(logits[0], params.top_k), params.temperature)
            u = philox.uniform(params.seed, i, rho, seq, philox.STREAM_DRAFT)
            y = sample_inverse_cdf(qi, u)
            trace.append(("draft", i, y, cdf_margin(qi, u, y)))
        y = int(forced.get(("draft", i), y))
        cand.append(y)
        if i > 1 and head is not None:
            s = accept_prob(head, hid[0])
            s_used.append(s)
            p_hat *= s
        stop = should_stop(p_hat, params.h)
        trace.append(("stop", i, int(stop), abs(1.0 - p_hat - params.h)))
        stop = bool(forced.get(("stop", i), stop))
        if k_forced is not None:
            continue                                     # the imposed count decides, not the rule
        if stop:
            break
        if params.eos_id >= 0 and y == params.eos_id:
            break
    K = len(cand)
    p_logits, _ = target.tail(x + cand, K + 1)
    q_logits = np.stack(q_rows) if q_rows else np.zeros((0, p_logits.shape[-1]))
    res = accept_resample(p_logits, q_logits, cand, K, temperature=params.temperature,
                          greedy=params.greedy, seed=params.seed, rnd=rho, seq=seq, forced=forced,
                          top_k=params.top_k)
    for i in range(1, K + 1):
        trace.append(("accept", i, int(res["flags"][i - 1]),
                      res["ratio"][i - 1] if params.greedy else abs(res["r"][i - 1] - res["ratio"][i - 1])))
    trace.append(("token", res["n"] + 1, res["token"], res["margin"]))
    n = res["n"]
    return dict(K=K, n=n, cand=cand, tokens=cand[:n] + [res["token"]], q_logits=q_logits,
                p_logits=p_logits, s=s_used, p_hat=p_hat, flags=res["flags"], trace=trace)


def oracle_generate(target_w: ModelWeights, draft_w: ModelWeights, head: Optional[HeadWeights], prompt,
                    params: Params, max_new: int, k_max: int, max_seq: int, seq: int = 0,
                    cached: bool = False, forced: Optional[Callable[[int], dict]] = None):
    """Draft-verify-correct rounds until max_new tokens (or EOS).  A round may
    overshoot max_new; the output is truncated and N counts kept tokens only.

    Returns (tokens generated, Stats, per-round result dicts).
    """
    mk = Cached if cached else Recompute
    target, draft = mk(target_w), mk(draft_w)
    x = [int(t) for t in prompt]
    out: List[int] = []
    stats = Stats()
    rounds = []
    rho = 0
    done = False
    while len(out) < max_new and not done:
        res = oracle_round(target, draft, head, x, rho, params, k_max, max_seq, seq,
                           forced(rho) if forced else None)
        new = res["tokens"]
        if params.eos_id >= 0 and params.eos_id in new:
            new = new[: new.index(params.eos_id) + 1]
            done = True
        kept = new[: max_new - len(out)]
        out += kept
        x += res["tokens"]
        stats.N += len(kept)
        stats.N_draft += res["K"]
        stats.N_target += 1
        stats.N_discarded += res["K"] - res["n"]
        stats.K_hist.append(res["K"])
        stats.n_hist.append(res["n"])
        rounds.append(res)
        rho += 1
    return out, stats, rounds


def target_greedy_generate(target_w: ModelWeights, prompt, max_new: int, eos_id: int = -1) -> List[int]:
    """The plain definition: the target's own autoregressive greedy tokens
    X_1..X_N (Sec. 4.1), one full forward per token, no draft model anywhere."""
    x = [int(t) for t in prompt]
    out: List[int] = []
    for _ in range(max_new):
        logits, _ = forward_full(target_w, x)
        t = argmax_lowest(logits[-1])
        out.append(t)
        x.append(t)
        if eos_id >= 0 and t == eos_id:
            break
    return out


def hindsight_counts(target_w: ModelWeights, draft_w: ModelWeights, prompt, N: int) -> dict:
    """The hindsight-optimal stopping policy of greedy speculative decoding (Sec. 4.1, Theorem 1).

    X_1..X_N are the target's own greedy tokens; Y_i = argmax q(. | prompt, X_1..X_{i-1}) is the
    draft's greedy token given the target's partial generation; S = {i : Y_i != X_i}.  Stopping
    right before every i in S discards nothing and calls the target once per element of S (that
    call emits X_i) plus once for the tokens behind the last disagreement.

    Returns dict(X, Y, S (1-based), plan, N_draft, N_target, N_discarded = 0), where plan[r] is the
    number of candidates the policy drafts in round r (0 when two disagreements are adjacent: the
    target simply takes a step).  N_target is the theorem's |S| + 1, except that when X_N itself is
    a disagreement nothing is left for a last round and the count is |S|.
    """
    prompt = [int(t) for t in prompt]
    X = target_greedy_generate(target_w, prompt, N)
    # row P-1+j of the draft's forward over (prompt, X_1..X_{N-1}) is conditioned on prompt, X_1..X_j
    logits, _ = forward_full(draft_w, prompt + X[:-1])
    P = len(prompt)
    Y = [argmax_lowest(logits[P - 1 + j]) for j in range(N)]
    S = [i for i in range(1, N + 1) if Y[i - 1] != X[i - 1]]
    plan, pos = [], 0                    # pos = tokens emitted so far
    for i in S + ([] if S and S[-1] == N else [N + 1]):
        # candidates Y_{pos+1}..Y_{i-1} all agree; the target's call emits X_i (or, in the last
        # round, the bonus token X_N after N - pos - 1 accepted candidates)
        k = min(i, N) - pos - 1
        plan.append(k)
        pos += k + 1
    assert pos == N
    return dict(X=X, Y=Y, S=S, plan=plan, N_draft=sum(plan), N_target=len(plan), N_discarded=0)
