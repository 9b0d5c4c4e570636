"""Pins for oracle/sampling.py against what the paper and probability fix:
unbiasedness of rejection sampling (Appendix C), the per-token acceptance
probability sum_v min(p_v, q_v) (Sec. 4.3), perfect alignment (Appendix B.1),
and the constant-alpha expectation (1 - alpha^(K+1)) / (1 - alpha)."""
import os

import numpy as np
from scipy import stats

from oracle import philox, sampling

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand_dist(rng, v, sharp=1.5):
    return rng.normal(0, sharp, size=v)


def _draw_candidates(q_logits, seed, rnd):
    """Candidates y_i ~ q_i, each with its own uniform (stream 0), as the round does."""
    q = sampling.softmax(q_logits)
    return [sampling.sample_inverse_cdf(q[i], philox.uniform(seed, i + 1, rnd, 0, philox.STREAM_DRAFT))
            for i in range(q.shape[0])]


def test_inverse_cdf_brute_force():
    rng = np.random.default_rng(0)
    for _ in range(300):
        v = int(rng.integers(1, 9))
        f = rng.random(v) * (rng.random(v) > 0.3)
        if f.sum() == 0:
            f[rng.integers(v)] = 1.0
        u = rng.random()
        # definition, spelled with exact rationals over the partial sums
        acc, want = 0.0, None
        for i in range(v):
            acc += f[i]
            if acc > u * f.sum() and want is None:
                want = i
        got = sampling.sample_inverse_cdf(f, u)
        assert f[got] > 0
        if want is not None:
            assert got == want


def test_inverse_cdf_frequencies_match_weights():
    f = np.array([0.1, 0.0, 0.4, 0.2, 0.3])
    us = philox.uniform_np(3, np.arange(1, 40001), 0, 0, 0)
    counts = np.bincount([sampling.sample_inverse_cdf(f, u) for u in us], minlength=5)
    assert counts[1] == 0
    keep = f > 0
    assert stats.chisquare(counts[keep], f[keep] / f.sum() * counts.sum()).pvalue > 1e-3


def test_argmax_ties_go_to_lowest_id():
    assert sampling.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0])) == 1


def test_softmax_is_scipy_softmax():
    from scipy.special import softmax as sp_softmax
    x = np.random.default_rng(1).normal(0, 3, size=(4, 37))
    np.testing.assert_allclose(sampling.softmax(x, 0.7), sp_softmax(x / 0.7, axis=-1), rtol=1e-13)


def test_emitted_tokens_follow_target_distribution():
    """Chained rejection sampling is unbiased: with context-free rows, the token
    emitted at position j (when the round reaches it) is distributed as p_j."""
    rng = np.random.default_rng(2)
    V, K, trials = 8, 3, 30000
    p_logits = _rand_dist(rng, (K + 1) * V).reshape(K + 1, V)
    q_logits = p_logits[:K] + rng.normal(0, 1.0, size=(K, V))
    p = sampling.softmax(p_logits)
    counts = np.zeros((K + 1, V))
    for t in range(trials):
        cand = _draw_candidates(q_logits, 11, t)
        res = sampling.accept_resample(p_logits, q_logits, cand, K, seed=11, rnd=t)
        emitted = cand[: res["n"]] + [res["token"]]
        for j, tok in enumerate(emitted):
            counts[j, tok] += 1
    for j in range(K + 1):
        tot = counts[j].sum()
        if tot < 2000:
            continue
        assert stats.chisquare(counts[j], p[j] * tot).pvalue > 1e-3, j
    assert counts[0].sum() == trials


def test_acceptance_rate_is_sum_min_p_q_and_residual_histogram():
    rng = np.random.default_rng(3)
    V, trials = 12, 30000
    p_logits = _rand_dist(rng, 2 * V).reshape(2, V)
    q_logits = p_logits[:1] + rng.normal(0, 1.0, size=(1, V))
    p, q = sampling.softmax(p_logits), sampling.softmax(q_logits)
    alpha = np.minimum(p[0], q[0]).sum()
    acc = 0
    resid = np.zeros(V)
    for t in range(trials):
        cand = _draw_candidates(q_logits, 5, t)
        res = sampling.accept_resample(p_logits, q_logits, cand, 1, seed=5, rnd=t)
        acc += res["n"]
        if res["n"] == 0:
            resid[res["token"]] += 1
    se = np.sqrt(alpha * (1 - alpha) / trials)
    assert abs(acc / trials - alpha) < 4 * se
    want = np.maximum(p[0] - q[0], 0)
    want = want / want.sum()
    assert (resid[want == 0] == 0).all()
    keep = want > 0
    assert stats.chisquare(resid[keep], want[keep] * resid.sum()).pvalue > 1e-3


def test_perfect_alignment_accepts_everything():
    rng = np.random.default_rng(4)
    V, K = 16, 6
    logits = _rand_dist(rng, (K + 1) * V).reshape(K + 1, V)
    for t in range(300):
        cand = _draw_candidates(logits[:K], 1, t)
        res = sampling.accept_resample(logits, logits[:K], cand, K, seed=1, rnd=t)
        assert res["n"] == K and res["flags"].all()


def test_constant_alpha_expected_tokens_per_round():
    """q = (1/2, 1/2), p = (1/2 + d, 1/2 - d) gives acceptance 1 - d at every
    position, whatever was drawn; mean(n + 1) must hit the closed form."""
    for line in open(os.path.join(GOLD, "constant_alpha.txt")):
        line = line.split("#")[0].split()
        if len(line) != 3:
            continue
        alpha, K, want = float(line[0]), int(line[1]), float(line[2])
        d = 1 - alpha
        with np.errstate(divide="ignore"):
            p_logits = np.log(np.tile([0.5 + d, 0.5 - d], (K + 1, 1)))
        q_logits = np.log(np.tile([0.5, 0.5], (K, 1)))
        trials, tot, sq = 12000, 0, 0
        for t in range(trials):
            cand = _draw_candidates(q_logits, 21, t)
            n1 = sampling.accept_resample(p_logits, q_logits, cand, K, seed=21, rnd=t)["n"] + 1
            tot += n1
            sq += n1 * n1
        mean = tot / trials
        se = np.sqrt((sq / trials - mean * mean) / trials)
        assert abs(mean - want) < 4 * se, (alpha, K, mean, want)


def test_greedy_accepts_up_to_first_mismatch():
    p_logits = np.array([[0, 5, 1], [4, 0, 1], [0, 1, 9], [7, 0, 0]], dtype=float)
    q_logits = np.zeros((3, 3))
    res = sampling.accept_resample(p_logits, q_logits, [1, 0, 2], 3, greedy=True)
    assert res["n"] == 3 and res["token"] == 0
    res = sampling.accept_resample(p_logits, q_logits, [1, 2, 2], 3, greedy=True)
    assert res["n"] == 1 and res["token"] == 0 and list(res["flags"]) == [1, 0, 1]


def test_accept_uses_ratio_p_over_q_orientation():
    """A candidate with p(y) >= q(y) is always accepted; one with p(y) = 0 never."""
    p_logits = np.log(np.array([[0.9, 0.1 - 1e-12, 1e-12], [1 / 3, 1 / 3, 1 / 3]]))
    q_logits = np.log(np.array([[0.2, 0.4, 0.4]]))
    for t in range(200):
        assert sampling.accept_resample(p_logits, q_logits, [0], 1, seed=2, rnd=t)["n"] == 1
        res = sampling.accept_resample(p_logits, q_logits, [2], 1, seed=2, rnd=t)
        assert res["n"] == 0 and res["token"] == 0       # residual mass sits on token 0 only


def test_top_k_warp_matches_torch_topk_and_keeps_ties():
    import torch
    rng = np.random.default_rng(7)
    x = rng.normal(size=(5, 40))
    for k in (1, 3, 10, 39):
        got = sampling.warp_top_k(x, k)
        idx = torch.topk(torch.from_numpy(x), k, dim=-1).indices.numpy()
        want = np.full_like(x, -np.inf)
        np.put_along_axis(want, idx, np.take_along_axis(x, idx, -1), -1)
        np.testing.assert_array_equal(got, want)
    assert sampling.warp_top_k(x, 0) is not None and np.array_equal(sampling.warp_top_k(x, 0), x)
    assert np.array_equal(sampling.warp_top_k(x, 40), x) and np.array_equal(sampling.warp_top_k(x, 99), x)
    tied = np.array([[3.0, 1.0, 3.0, 2.0, 3.0]])
    assert np.isfinite(sampling.warp_top_k(tied, 2)).sum() == 3       # all three maxima survive


def test_top_k_rounds_are_unbiased_for_the_warped_target():
    """With top-k warping on both models the emitted token follows the WARPED target
    distribution, and never leaves the target's top-k set."""
    rng = np.random.default_rng(8)
    V, K, k, trials = 12, 2, 4, 30000
    p_logits = _rand_dist(rng, (K + 1) * V).reshape(K + 1, V)
    q_logits = p_logits[:K] + rng.normal(0, 1.0, size=(K, V))
    pw = sampling.softmax(sampling.warp_top_k(p_logits, k))
    qw = sampling.softmax(sampling.warp_top_k(q_logits, k))
    counts = np.zeros((K + 1, V))
    for t in range(trials):
        cand = [sampling.sample_inverse_cdf(qw[i], philox.uniform(13, i + 1, t, 0, philox.STREAM_DRAFT)) for i in range(K)]
        res = sampling.accept_resample(p_logits, q_logits, cand, K, seed=13, rnd=t, top_k=k)
        for j, tok in enumerate(cand[: res["n"]] + [res["token"]]):
            counts[j, tok] += 1
    for j in range(K + 1):
        tot = counts[j].sum()
        assert (counts[j][pw[j] == 0] == 0).all()
        if tot < 2000:
            continue
        keep = pw[j] > 0
        assert stats.chisquare(counts[j][keep], pw[j][keep] * tot).pvalue > 1e-3, j
