"""Pins for oracle/rounds.py: greedy speculative decoding reproduces the target's
own greedy tokens (Sec. 4.1); the counter identity of Sec. 3.2; fixed K as the
h >= 1 special case (Appendix D.4); unbiasedness of a whole sampled round; cached
and recomputing forwards give the same rounds."""
import numpy as np
import torch
from scipy import stats

from oracle import rounds as R
from oracle import sampling
from oracle.model import forward_full
from paper_2405_19715_amd import synth
from tests._util import oracle_head, oracle_model

SHAPE = synth.ModelShape(n_layers=2, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48, vocab=40)


def _pair(seed=0, perturb=0.05, std=0.25):
    t = synth.make_model(SHAPE, seed, dtype=torch.float64, std=std)
    d = synth.make_perturbed_draft(t, 1, seed + 1, std=perturb)
    h = synth.make_head([SHAPE.d_model, 8, 1], seed + 2, dtype=torch.float64, std=0.3)
    return oracle_model(t), oracle_model(d), oracle_head(h)


def test_greedy_rounds_equal_target_only_greedy_decoding():
    tw, dw, hw = _pair()
    prompt = synth.make_prompt(6, SHAPE.vocab, 1)
    want = R.target_greedy_generate(tw, prompt, 24)
    for h, k_max in [(0.7, 8), (1.0, 4), (-1.0, 8), (0.3, 3)]:
        got, st, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=h, greedy=True), 24, k_max, 64)
        assert got == want, (h, k_max)
        assert st.N == 24


def test_greedy_identity_with_unrelated_draft():
    tw, _, hw = _pair(seed=3)
    dw = oracle_model(synth.make_model(SHAPE, 99, dtype=torch.float64, std=0.25))
    prompt = synth.make_prompt(5, SHAPE.vocab, 2)
    want = R.target_greedy_generate(tw, prompt, 12)
    got, st, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=0.9, greedy=True), 12, 6, 64)
    assert got == want


def test_counter_identity_and_fixed_k_special_case():
    tw, dw, hw = _pair(seed=5)
    prompt = synth.make_prompt(6, SHAPE.vocab, 3)
    for h in (0.3, 0.7, 1.0):
        _, st, rounds = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=h, seed=4), 30, 5, 200)
        over = sum(len(r["tokens"]) for r in rounds) - st.N          # truncation of the last round
        assert st.N_draft + st.N_target == st.N + over + st.N_discarded
        assert 0 <= over <= 5
        for r in rounds:
            assert 0 <= r["n"] <= r["K"] <= 5 and len(r["tokens"]) == r["n"] + 1
        if h >= 1.0:
            assert all(k == 5 for k in st.K_hist) and st.N_draft == 5 * st.N_target
    _, st, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=-0.5, seed=4), 10, 5, 200)
    assert all(k == 1 for k in st.K_hist)


def test_round_follows_the_stop_rule_on_its_own_head_outputs():
    from oracle.head import candidate_length
    tw, dw, hw = _pair(seed=6)
    prompt = synth.make_prompt(6, SHAPE.vocab, 4)
    for h in (0.2, 0.5, 0.8):
        _, _, rounds = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=h, seed=1), 20, 7, 200)
        for r in rounds:
            s = list(r["s"]) + [1.0] * 8
            assert r["K"] == candidate_length(s, h, 7)
            assert len(r["s"]) == r["K"] - 1          # nothing multiplied in at i = 1


def test_cache_capacity_caps_the_candidate_length():
    tw, dw, hw = _pair(seed=7)
    prompt = synth.make_prompt(6, SHAPE.vocab, 5)
    target, draft = R.Recompute(tw), R.Recompute(dw)
    r = R.oracle_round(target, draft, hw, prompt, 0, R.Params(h=1.0), 8, max_seq=10)
    assert r["K"] == 3                                   # 6 + K + 1 <= 10
    try:
        R.oracle_round(target, draft, hw, prompt, 0, R.Params(h=1.0), 8, max_seq=7)
        assert False
    except OverflowError:
        pass


def test_eos_stops_drafting_and_generation():
    tw, dw, hw = _pair(seed=8)
    prompt = synth.make_prompt(6, SHAPE.vocab, 6)
    base, _, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=1.0, greedy=True), 16, 4, 200)
    eos = base[5]
    first = base.index(eos)
    got, st, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=1.0, greedy=True, eos_id=eos), 16, 4, 200)
    assert got == base[: first + 1]


def test_cached_mode_equals_recompute_mode():
    tw, dw, hw = _pair(seed=9)
    prompt = synth.make_prompt(7, SHAPE.vocab, 7)
    for greedy in (False, True):
        p = R.Params(h=0.6, greedy=greedy, seed=3)
        a, sa, _ = R.oracle_generate(tw, dw, hw, prompt, p, 20, 6, 200, cached=False)
        b, sb, _ = R.oracle_generate(tw, dw, hw, prompt, p, 20, 6, 200, cached=True)
        assert a == b and sa.K_hist == sb.K_hist and sa.n_hist == sb.n_hist


def test_first_sampled_token_follows_target_distribution():
    """Whole round, many seeds: the first emitted token is a draw from the
    target's next-token distribution (unbiasedness, Appendix C)."""
    tw, dw, hw = _pair(seed=10, perturb=0.15)
    prompt = synth.make_prompt(4, SHAPE.vocab, 8)
    p = sampling.softmax(forward_full(tw, prompt)[0][-1])
    target, draft = R.Cached(tw), R.Cached(dw)
    counts = np.zeros(SHAPE.vocab)
    trials = 4000
    for seed in range(trials):
        r = R.oracle_round(target, draft, hw, list(prompt), 0, R.Params(h=0.5, seed=seed), 3, 64)
        counts[r["tokens"][0]] += 1
    keep = p * trials > 5
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(p[keep], p[~keep].sum()) * trials
    assert stats.chisquare(obs, exp).pvalue > 1e-3


def _aligned_pair(seed, perturb):
    """A draft with all of the target's layers plus noise: agrees with the target on part of the tokens."""
    t = synth.make_model(SHAPE, seed, dtype=torch.float64, std=0.25)
    d = synth.make_perturbed_draft(t, SHAPE.n_layers, seed + 1, std=perturb)
    h = synth.make_head([SHAPE.d_model, 8, 1], seed + 2, dtype=torch.float64, std=0.3)
    return oracle_model(t), oracle_model(d), oracle_head(h)


def _play(tw, dw, hw, prompt, N, plan_of):
    """Greedy rounds with the candidate count of every round imposed by plan_of(tokens so far)."""
    target, draft = R.Recompute(tw), R.Recompute(dw)
    x, out, st, rho = list(prompt), [], R.Stats(), 0
    while len(out) < N:
        k = plan_of(len(out))
        r = R.oracle_round(target, draft, hw, x, rho, R.Params(greedy=True), 64, 512, forced={"K": k})
        assert r["K"] == k
        x += r["tokens"]
        out += r["tokens"]
        st.N_draft += k
        st.N_target += 1
        st.N_discarded += k - r["n"]
        rho += 1
    return out, st


def test_hindsight_policy_discards_nothing_and_calls_the_target_once_per_disagreement():
    """Sec. 4.1, Theorem 1, checked by playing the policy through the rounds: stopping right before
    every disagreement yields the target's own tokens with N_discarded = 0 and N_target = |S| + 1
    (|S| when the last token is itself a disagreement)."""
    seen_adjacent = seen_last = seen_open = False
    for seed, perturb in ((0, 0.02), (3, 0.08), (4, 0.03), (6, 0.05)):
        tw, dw, hw = _aligned_pair(seed, perturb)
        prompt = synth.make_prompt(6, SHAPE.vocab, seed)
        N = 20
        hs = R.hindsight_counts(tw, dw, prompt, N)
        X, S = hs["X"], hs["S"]
        assert X == R.target_greedy_generate(tw, prompt, N)
        # S by its definition, one draft forward per position (the function uses a single forward)
        for i in range(1, N + 1):
            yi = sampling.argmax_lowest(forward_full(dw, list(prompt) + X[: i - 1])[0][-1])
            assert (yi != X[i - 1]) == (i in S)
        last = bool(S) and S[-1] == N
        assert hs["N_target"] == len(S) + (0 if last else 1) and hs["N_discarded"] == 0
        assert hs["N_draft"] + hs["N_target"] == N          # Sec. 3.2's identity with nothing discarded
        seen_adjacent |= 0 in hs["plan"][:-1]
        seen_last |= last
        seen_open |= not last and hs["plan"][-1] > 0
        it = iter(hs["plan"])
        out, st = _play(tw, dw, hw, prompt, N, lambda pos: next(it))
        assert out == X
        assert (st.N_draft, st.N_target, st.N_discarded) == (hs["N_draft"], hs["N_target"], 0)
    # the cases cover a target step without candidates, a last token that is a disagreement, and a last
    # round that ends on the bonus token
    assert seen_adjacent and seen_last and seen_open


def test_no_stopping_policy_beats_hindsight_brute_force():
    """Every stopping policy on a short generation (all candidate counts in every round, by
    dynamic programming over the position with the rounds actually played): none discards less,
    none calls the target less often, so by the time decomposition of Sec. 3.2
    (T = T_0 + t_draft N_discarded + (t_target - t_draft) N_target) none is faster."""
    tw, dw, hw = _aligned_pair(0, 0.02)
    prompt = synth.make_prompt(6, SHAPE.vocab, 0)
    N = 14
    hs = R.hindsight_counts(tw, dw, prompt, N)
    assert 0 < len(hs["S"]) < N
    X = hs["X"]
    target, draft = R.Recompute(tw), R.Recompute(dw)
    gain = {}                                   # (pos, k) -> accepted candidates n of that round
    for pos in range(N):
        for k in range(0, N - pos):
            r = R.oracle_round(target, draft, hw, list(prompt) + X[:pos], 0, R.Params(greedy=True), 64, 512,
                               forced={"K": k})
            assert r["tokens"] == X[pos: pos + r["n"] + 1]
            gain[(pos, k)] = r["n"]
    best = {N: (0, 0)}                          # pos -> set of (N_target, N_discarded) reachable to the end
    frontier = {N: {(0, 0)}}
    for pos in range(N - 1, -1, -1):
        outs = set()
        for k in range(0, N - pos):
            n = gain[(pos, k)]
            for (nt, nd) in frontier[min(N, pos + n + 1)]:
                outs.add((nt + 1, nd + k - n))
        frontier[pos] = outs
    all_plans = frontier[0]
    assert min(nt for nt, _ in all_plans) == hs["N_target"]
    assert min(nd for _, nd in all_plans) == 0
    assert (hs["N_target"], 0) in all_plans
    t_d, t_t = 1.0, 4.8                          # the paper's ratio of forward times, about 0.0234 : 0.112
    cost = lambda nt, nd: t_d * N + t_d * nd + (t_t - t_d) * nt
    assert min(cost(nt, nd) for nt, nd in all_plans) == cost(hs["N_target"], 0)
