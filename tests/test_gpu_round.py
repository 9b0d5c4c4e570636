"""Parity of whole draft-verify-correct rounds (Algorithm 2) between the HIP path
and the oracle: free-running token streams on the tiny fp32 pair in greedy and
sampling mode, greedy identity with target-only decoding (Sec. 4.1), the counter
identity (Sec. 3.2), the fixed-K special case, and decision replay on bf16 pairs."""
import numpy as np
import pytest
import torch

from oracle import head as OH
from oracle import rounds as R
from oracle import sampling
from paper_2405_19715_amd import synth
from tests._parity import run_free_running
from tests._util import oracle_head, oracle_model

pytestmark = pytest.mark.gpu


def _cuda_model(m, share=None):
    out = dict(m)
    for k in ("tok_emb", "lm_head", "final_norm"):
        out[k] = share[k] if share is not None and m[k] is share["_src"][k] else m[k].cuda()
    out["layers"] = [{k: v.cuda() for k, v in lay.items()} for lay in m["layers"]]
    out["_src"] = m
    return out


def _cuda_head(h):
    out = dict(h)
    out["W"] = [w.cuda() for w in h["W"]]
    out["b"] = [b.cuda() for b in h["b"]]
    return out


def tiny_pair(seed=0):
    """The tiny fp32 pair: 2-layer target, draft = its first layer perturbed, shared
    embedding / LM head, head 256 -> 64 -> 1 with output bias logit(0.8)."""
    t = synth.make_model(synth.TINY_TARGET, seed, dtype=torch.float32)
    d = synth.make_perturbed_draft(t, 1, seed + 1, std=0.005)
    h = synth.make_head([256, 64, 1], seed + 2, dtype=torch.float32)
    return t, d, h


def _context(t, d, h, k_max, max_seq, batch=1):
    from paper_2405_19715_amd import binding as B
    tc = _cuda_model(t)
    dc = _cuda_model(d, share=tc)
    return B.Context(tc, dc, _cuda_head(h) if h is not None else None, batch=batch, max_seq=max_seq, k_max=k_max)


@pytest.mark.parametrize("greedy", [True, False])
def test_tiny_pair_free_running_parity(greedy):
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair()
    prompt = synth.make_prompt(64, 1024, 0)
    ctx = _context(t, d, h, k_max=8, max_seq=256)
    try:
        ctx.sd_prefill(0, prompt)
        op = R.Params(h=0.7, temperature=1.0, greedy=greedy, seed=0)
        gp = B.make_params(h=0.7, temperature=1.0, greedy=greedy, seed=0)
        toks, exempt, hist = run_free_running(ctx, oracle_model(t), oracle_model(d), oracle_head(h), prompt, op, gp,
                                              128, 8, 256)
        assert len(toks) == 128 and exempt <= 2
        assert max(k for k, _ in hist) <= 8
        st = ctx.sd_seq_state(0)
        assert st["P"] == 64 + sum(n + 1 for _, n in hist)
        assert st["kv_len_target"] == st["P"] - 1
    finally:
        ctx.close()


@pytest.mark.parametrize("top_k", [1, 8, 50])
def test_tiny_pair_free_running_parity_top_k(top_k):
    """Sampled rounds with top-k warping of both models (Appendix D.1)."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair()
    prompt = synth.make_prompt(48, 1024, 4)
    ctx = _context(t, d, h, k_max=8, max_seq=256)
    try:
        ctx.sd_prefill(0, prompt)
        op = R.Params(h=0.7, temperature=0.8, seed=9, top_k=top_k)
        gp = B.make_params(h=0.7, temperature=0.8, seed=9, top_k=top_k)
        toks, exempt, hist = run_free_running(ctx, oracle_model(t), oracle_model(d), oracle_head(h), prompt, op, gp,
                                              96, 8, 256)
        assert len(toks) == 96 and exempt <= 2
    finally:
        ctx.close()


@pytest.mark.parametrize("h,want_K", [(-0.5, 1), (0.0, 2), (1.0, 8)])
def test_degenerate_thresholds(h, want_K):
    """h < 0 stops after the first candidate (1 - p_hat = 0 > h before any prediction), h = 0
    after the second (the first prediction below 1), h >= 1 never (fixed K = K_max): free-running
    parity with the oracle at each, without and with the head (without it p_hat stays 1)."""
    from paper_2405_19715_amd import binding as B
    t, d, hd = tiny_pair()
    prompt = synth.make_prompt(30, 1024, 6)
    for head in (hd, None):
        ctx = _context(t, d, head, k_max=8, max_seq=192)
        try:
            ctx.sd_prefill(0, prompt)
            op = R.Params(h=h, temperature=1.0, greedy=False, seed=5)
            gp = B.make_params(h=h, temperature=1.0, greedy=False, seed=5)
            toks, exempt, hist = run_free_running(ctx, oracle_model(t), oracle_model(d),
                                                  oracle_head(head) if head is not None else None, prompt, op, gp,
                                                  40, 8, 192)
            assert exempt <= 1
            if head is not None or h < 0 or h >= 1:
                assert all(k == want_K for k, _ in hist), hist
            else:
                assert all(k == 8 for k, _ in hist), hist          # no head: p_hat = 1, 1 - p_hat = 0 is not > 0
        finally:
            ctx.close()


@pytest.mark.parametrize("greedy", [True, False])
def test_largest_supported_candidate_length(greedy):
    """K_max = 32, the largest the library takes, with h = 1 so that every round drafts all 32
    (Algorithm 1 with fixed K): 33 target rows, 65 softmax rows, 32 accept tests per round.  Tiny
    fp32 pair, free-running against the oracle."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair()
    prompt = synth.make_prompt(40, 1024, 2)
    ctx = _context(t, d, h, k_max=32, max_seq=320)
    try:
        ctx.sd_prefill(0, prompt)
        op = R.Params(h=1.0, temperature=1.0, greedy=greedy, seed=3)
        gp = B.make_params(h=1.0, temperature=1.0, greedy=greedy, seed=3)
        toks, exempt, hist = run_free_running(ctx, oracle_model(t), oracle_model(d), oracle_head(h), prompt, op, gp,
                                              96, 32, 320)
        assert len(toks) == 96 and exempt <= 2
        assert all(k == 32 for k, _ in hist)
    finally:
        ctx.close()


def test_largest_supported_candidate_length_bf16_rows():
    """The same on a bf16 pair: 33 target rows is more than the streaming GEMM takes, so the target
    pass goes through the tiled kernel with K slices and attention through three query-tile groups
    per kv head; rows against the oracle's teacher-forced forward, decisions replayed."""
    from paper_2405_19715_amd import binding as B
    from oracle.model import forward_full
    t, d, h = _bf16_pair()
    prompt = synth.make_prompt(70, 2048, 15)
    ctx = _context(t, d, h, k_max=32, max_seq=256)
    try:
        ctx.sd_prefill(0, prompt)
        x = list(prompt)
        tw, dw = oracle_model(t), oracle_model(d)
        for rho in range(2):
            g = ctx.specdec_round(B.make_params(h=1.0, seed=7))[0]
            K = g["K"]
            assert K == 32
            q, p, _ = ctx.sd_last_round_rows(0, K)
            q, p = q.numpy(), p.numpy()
            want_p = forward_full(tw, x + g["cand"])[0][-(K + 1):]
            want_q = forward_full(dw, x + g["cand"][:-1])[0][-K:]
            for got, want in ((p, want_p), (q, want_q)):
                err = (np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()
                assert err < 2e-2, (rho, err)
            o = sampling.accept_resample(p, q, g["cand"], K, seed=7, rnd=rho)
            if o["n"] != g["n"]:
                i = min(o["n"], g["n"]) + 1
                assert abs(o["r"][i - 1] - o["ratio"][i - 1]) < 1e-3
                o = sampling.accept_resample(p, q, g["cand"], K, seed=7, rnd=rho,
                                             forced={("accept", i): 1 if g["n"] >= i else 0})
            assert o["n"] == g["n"]
            assert o["token"] == g["tokens"][-1] or o["margin"] < 1e-5
            x += g["tokens"]
    finally:
        ctx.close()


def test_greedy_generate_equals_target_only_greedy_and_counters():
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=3)
    prompt = synth.make_prompt(20, 1024, 5)
    want = R.target_greedy_generate(oracle_model(t), prompt, 40)
    for hh, k_max in [(0.7, 8), (1.0, 4), (-1.0, 8)]:
        ctx = _context(t, d, h, k_max=k_max, max_seq=128)
        try:
            ctx.sd_prefill(0, prompt)
            seqs, st = ctx.specdec_generate(B.make_params(h=hh, greedy=True), 40)
            assert seqs[0] == want, (hh, k_max)
            assert st["N"] == 40
            # whole rounds satisfy N_draft + N_target = N + N_discarded; the last round may overshoot
            over = st["N_draft"] + st["N_target"] - st["N"] - st["N_discarded"]
            assert 0 <= over <= k_max
            if hh >= 1.0:
                assert st["N_draft"] == k_max * st["N_target"]
            if hh < 0:
                assert st["N_draft"] == st["N_target"]
        finally:
            ctx.close()


def test_hindsight_disagreement_set_from_hip_greedy_tokens_matches_oracle():
    """Sec. 4.1, Theorem 1 on the HIP path: X = the greedy tokens the rounds emit, Y_i = argmax of
    the draft's teacher-forced row conditioned on (prompt, X_<i) (sd_forward on the draft), S where
    they differ; S and the counts it implies must be the oracle's.  Any actual run calls the target
    at least that often."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=3)
    for perturb_seed, n_prompt, N, std in ((4, 20, 72, 0.002), (9, 33, 64, 0.003)):
        # all of the target's layers plus a little noise: agrees with the target on part of the tokens
        d = synth.make_perturbed_draft(t, 2, perturb_seed, std=std)
        prompt = synth.make_prompt(n_prompt, 1024, perturb_seed)
        hs = R.hindsight_counts(oracle_model(t), oracle_model(d), prompt, N)
        assert 2 < len(hs["S"]) < N - 2 and max(hs["plan"]) >= 2, hs["S"]
        ctx = _context(t, d, h, k_max=8, max_seq=192)
        try:
            ctx.sd_prefill(0, prompt)
            seqs, st = ctx.specdec_generate(B.make_params(h=0.7, greedy=True), N)
            X = seqs[0]
            assert X == hs["X"]
            # teacher-forced draft rows: feeding prompt[-1], X_1 .. X_{N-1} from cache position n_prompt - 1
            ctx.sd_prefill(0, prompt)
            fed = [prompt[-1]] + X[:-1]
            Y = []
            for s0 in range(0, N, 32):
                rows = ctx.sd_forward(1, 0, n_prompt - 1 + s0, fed[s0:s0 + 32]).numpy()
                Y += [int(np.argmax(r)) for r in rows]
            S = [i + 1 for i in range(N) if Y[i] != X[i]]
            assert S == hs["S"]
            n_target = len(S) + (0 if S and S[-1] == N else 1)
            assert n_target == hs["N_target"] and N - n_target == hs["N_draft"]
            assert st["N_target"] >= n_target and st["N_discarded"] >= 0
        finally:
            ctx.close()


def test_sampled_generate_matches_oracle_generate_and_resumes():
    """specdec_generate(N) equals the oracle's stream, and equals generate(N1) followed
    by generate(N - N1) when N1 ends on a round boundary (counter-based uniforms)."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=7)
    prompt = synth.make_prompt(16, 1024, 9)
    op = R.Params(h=0.5, seed=11)
    want, ost, rounds = R.oracle_generate(oracle_model(t), oracle_model(d), oracle_head(h), prompt, op, 48, 6, 128,
                                          cached=True)
    ctx = _context(t, d, h, k_max=6, max_seq=128)
    try:
        ctx.sd_prefill(0, prompt)
        seqs, st = ctx.specdec_generate(B.make_params(h=0.5, seed=11), 48)
        assert seqs[0] == want
        assert (st["N"], st["N_draft"], st["N_target"], st["N_discarded"]) == (ost.N, ost.N_draft, ost.N_target,
                                                                              ost.N_discarded)
        n1 = sum(len(r["tokens"]) for r in rounds[:3])
        ctx.sd_prefill(0, prompt)
        a, _ = ctx.specdec_generate(B.make_params(h=0.5, seed=11), n1)
        b, _ = ctx.specdec_generate(B.make_params(h=0.5, seed=11), 48 - n1)
        assert a[0] + b[0] == want
    finally:
        ctx.close()


def test_cache_capacity_and_bad_arguments():
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=1)
    for bad_seq in (100, 12352):                            # not a multiple of 64; more than an fp32 model takes
        with pytest.raises(B.SpecDecError) as e:
            _context(t, d, h, k_max=8, max_seq=bad_seq)
        assert e.value.status == B.SD_EINVAL
    ctx = _context(t, d, h, k_max=8, max_seq=64)
    try:
        with pytest.raises(B.SpecDecError) as e:
            ctx.sd_prefill(0, [5000])                       # token id outside the vocabulary
        assert e.value.status == B.SD_ERANGE
        with pytest.raises(B.SpecDecError) as e:
            ctx.sd_prefill(0, list(range(63)))              # n + 2 > max_seq
        assert e.value.status == B.SD_ERANGE
        prompt = synth.make_prompt(58, 1024, 2)
        ctx.sd_prefill(0, prompt)
        for bad in (B.make_params(top_k=-1), B.make_params(temperature=0.0)):
            with pytest.raises(B.SpecDecError) as e:
                ctx.specdec_round(bad)
            assert e.value.status == B.SD_EINVAL and ctx.sd_seq_state(0)["P"] == 58
        r = ctx.specdec_round(B.make_params(h=1.0, seed=1))[0]
        assert r["K"] == 64 - 58 - 1                        # cap = max_seq - P - 1
        # rounds go on until the cache is full, then the call reports it and changes nothing
        while True:
            st = ctx.sd_seq_state(0)
            if 64 - st["P"] - 1 < 1:
                break
            ctx.specdec_round(B.make_params(h=1.0, seed=1))
        before = ctx.sd_seq_state(0)
        with pytest.raises(B.SpecDecError) as e:
            ctx.specdec_round(B.make_params(h=1.0, seed=1))
        assert e.value.status == B.SD_ERANGE and ctx.sd_seq_state(0) == before
    finally:
        ctx.close()


def _bf16_pair(wide=False):
    if wide:
        # widths of 2048 / 4096: up to 8 rows go through the row-stripe GEMM and its fused epilogues (the models'
        # matrices, the acceptance head's layers with their row gather, the LM head)
        ts = synth.ModelShape(2, 2048, 16, 2, 128, 4096, 2048)
        ds = synth.ModelShape(1, 2048, 16, 16, 128, 2048, 2048)
        dims, std = [2048, 2048, 2048, 1], 0.02
    else:
        ts = synth.ModelShape(2, 512, 8, 1, 64, 640, 2048)
        ds = synth.ModelShape(1, 256, 2, 2, 128, 384, 2048)
        dims, std = [256, 256, 256, 256, 1], 0.04
    t = synth.make_model(ts, 20, dtype=torch.bfloat16, std=std)
    d = synth.make_model(ds, 21, dtype=torch.bfloat16, std=std)
    h = synth.make_head(dims, 22, dtype=torch.bfloat16, residual=True, std=std)
    return t, d, h


@pytest.mark.parametrize("greedy", [False, True])
def test_bf16_pair_decision_replay(greedy):
    """bf16 models: feed the HIP path's own fp32 logits rows and head outputs of each
    round to the oracle's stop rule and accept / resample step: K, n and y' must match
    exactly (same exemptions as above)."""
    from paper_2405_19715_amd import binding as B
    from oracle import philox
    t, d, h = _bf16_pair()
    prompt = synth.make_prompt(40, 2048, 3)
    k_max, hh, seed = 16, 0.9, 5
    ctx = _context(t, d, h, k_max=k_max, max_seq=256)
    try:
        ctx.sd_prefill(0, prompt)
        gp = B.make_params(h=hh, greedy=greedy, seed=seed)
        exempt = 0
        Ks = []
        for rho in range(12):
            g = ctx.specdec_round(gp)[0]
            K = g["K"]
            Ks.append(K)
            q, p, s = ctx.sd_last_round_rows(0, K)
            q, p, s = q.numpy(), p.numpy(), s.numpy()
            # stop rule on the head outputs the HIP path used
            want_K = OH.candidate_length(list(s.astype(np.float64)) + [1.0] * 40, hh, k_max)
            if want_K != K:
                ph = np.cumprod(np.concatenate([[1.0], s.astype(np.float64)]))
                assert np.min(np.abs(1 - ph - hh)) < 1e-5
                exempt += 1
            # candidates: inverse CDF / argmax on the HIP path's own draft rows
            for i in range(1, K + 1):
                if greedy:
                    y = sampling.argmax_lowest(q[i - 1])
                    ok = y == g["cand"][i - 1] or sampling.top2_gap(q[i - 1]) < 1e-6
                else:
                    qi = sampling.softmax(q[i - 1])
                    u = philox.uniform(seed, i, rho, 0, philox.STREAM_DRAFT)
                    y = sampling.sample_inverse_cdf(qi, u)
                    ok = y == g["cand"][i - 1] or sampling.cdf_margin(qi, u, y) < 1e-5
                assert ok, (rho, i)
                exempt += int(y != g["cand"][i - 1])
            o = sampling.accept_resample(p, q, g["cand"], K, greedy=greedy, seed=seed, rnd=rho)
            if o["n"] != g["n"]:
                i = min(o["n"], g["n"]) + 1
                assert not greedy and abs(o["r"][i - 1] - o["ratio"][i - 1]) < 1e-3
                o = sampling.accept_resample(p, q, g["cand"], K, greedy=greedy, seed=seed, rnd=rho,
                                             forced={("accept", i): 1 if g["n"] >= i else 0})
                exempt += 1
            assert o["n"] == g["n"]
            if o["token"] != g["tokens"][-1]:
                assert o["margin"] < 1e-5
                exempt += 1
            assert g["tokens"][:-1] == g["cand"][: g["n"]]
        assert exempt <= 3
        assert min(Ks) >= 2 and max(Ks) <= k_max
    finally:
        ctx.close()


def test_bf16_round_logits_match_oracle_forward():
    """Teacher-forced check of a real round: replay the HIP path's tokens through the
    oracle's fp64 forward and compare the target rows p_1..p_{K+1} and draft rows
    q_1..q_K the round used (row-wise max-norm relative error)."""
    from paper_2405_19715_amd import binding as B
    from oracle.model import forward_full
    t, d, h = _bf16_pair()
    prompt = synth.make_prompt(33, 2048, 8)
    ctx = _context(t, d, h, k_max=16, max_seq=256)
    try:
        ctx.sd_prefill(0, prompt)
        x = list(prompt)
        tw, dw = oracle_model(t), oracle_model(d)
        for rho in range(4):
            g = ctx.specdec_round(B.make_params(h=0.8, seed=2))[0]
            K = g["K"]
            q, p, _ = ctx.sd_last_round_rows(0, K)
            want_p = forward_full(tw, x + g["cand"])[0][-(K + 1):]
            want_q = forward_full(dw, x + g["cand"][:-1])[0][-K:]
            for got, want in ((p.numpy(), want_p), (q.numpy(), want_q)):
                err = (np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()
                assert err < 2e-2, (rho, err)
            x += g["tokens"]
    finally:
        ctx.close()


def test_long_context_batch_logits_match_oracle_forward():
    """Eight sequences with 600-1000 tokens of context decoded together: ten to sixteen key
    blocks per sequence, target rows packed per sequence (ragged K).  The rows
    p_1..p_{K+1} and q_1..q_K of every sequence against the oracle's teacher-forced forward."""
    from paper_2405_19715_amd import binding as B
    from oracle.model import forward_full
    ts = synth.ModelShape(1, 256, 32, 8, 64, 384, 2048)      # grouped queries, 4 per kv head
    ds = synth.ModelShape(1, 256, 32, 32, 64, 384, 2048)     # one kv head per query head
    t = synth.make_model(ts, 30, dtype=torch.bfloat16, std=0.04)
    d = synth.make_model(ds, 31, dtype=torch.bfloat16, std=0.04)
    h = synth.make_head([256, 256, 1], 32, dtype=torch.bfloat16, residual=True, std=0.04)
    Bn, seed = 8, 4
    lens = [1000, 640, 873, 702, 991, 600, 935, 777]
    prompts = [synth.make_prompt(lens[b], 2048, 70 + b) for b in range(Bn)]
    ctx = _context(t, d, h, k_max=16, max_seq=1088, batch=Bn)
    try:
        for b in range(Bn):
            ctx.sd_prefill(b, prompts[b])
        tw, dw = oracle_model(t), oracle_model(d)
        xs = [list(p) for p in prompts]
        seen_K = set()
        for rho in range(2):
            res = ctx.specdec_round(B.make_params(h=0.8, seed=seed))
            for b in range(Bn):
                g = res[b]
                K = g["K"]
                seen_K.add(K)
                q, p, _ = ctx.sd_last_round_rows(b, K)
                want_p = forward_full(tw, xs[b] + g["cand"])[0][-(K + 1):]
                want_q = forward_full(dw, xs[b] + g["cand"][:-1])[0][-K:]
                for got, want in ((p.numpy(), want_p), (q.numpy(), want_q)):
                    err = (np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()
                    assert err < 2e-2, (rho, b, err)
                xs[b] += g["tokens"]
        assert len(seen_K) > 1
    finally:
        ctx.close()


def test_batch_of_sequences_matches_single_sequence_runs():
    """Two sequences decoded together give the streams each gives alone (per-sequence
    stop rule, ragged K, per-sequence rollback; the sequence id keys the uniforms)."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=4)
    prompts = [synth.make_prompt(12, 1024, 1), synth.make_prompt(30, 1024, 2)]
    tw, dw, hw = oracle_model(t), oracle_model(d), oracle_head(h)
    want = [R.oracle_generate(tw, dw, hw, prompts[b], R.Params(h=0.6, seed=3), 24, 6, 128, seq=b, cached=True)[0]
            for b in range(2)]
    ctx = _context(t, d, h, k_max=6, max_seq=128, batch=2)
    try:
        for b in range(2):
            ctx.sd_prefill(b, prompts[b])
        seqs, st = ctx.specdec_generate(B.make_params(h=0.6, seed=3), 24)
        assert seqs == want
    finally:
        ctx.close()


def _ragged_batch_replay(Bn, k_max, hs, seed, max_exempt, check_rows=0, wide=False):
    """Bn sequences with different prompt lengths decoded together on a bf16 pair, one round per
    threshold in `hs`: every sequence's K, candidates, n and y' replayed by the oracle on the HIP
    path's own rows, and the sequence state stays consistent; for the first `check_rows` sequences
    the rows themselves against the oracle's teacher-forced forward.  Returns the set of K seen."""
    from paper_2405_19715_amd import binding as B
    from oracle import philox
    from oracle.model import forward_full
    t, d, h = _bf16_pair(wide)
    tw, dw = oracle_model(t), oracle_model(d)
    g0 = torch.Generator().manual_seed(123)
    lens = torch.randint(20, 90, (Bn,), generator=g0).tolist()
    prompts = [synth.make_prompt(lens[b], 2048, 50 + b) for b in range(Bn)]
    ctx = _context(t, d, h, k_max=k_max, max_seq=256, batch=Bn)
    try:
        for b in range(Bn):
            ctx.sd_prefill(b, prompts[b])
        P = list(lens)
        xs = [list(pr) for pr in prompts]
        exempt = 0
        seen_K = set()
        for rho, hh in enumerate(hs):
            res = ctx.specdec_round(B.make_params(h=hh, seed=seed))
            for b in range(Bn):
                g = res[b]
                K = g["K"]
                seen_K.add(K)
                q, p, s = ctx.sd_last_round_rows(b, K)
                q, p, s = q.numpy(), p.numpy(), s.numpy()
                if b < check_rows:
                    want_p = forward_full(tw, xs[b] + g["cand"])[0][-(K + 1):]
                    want_q = forward_full(dw, xs[b] + g["cand"][:-1])[0][-K:]
                    for got, want in ((p, want_p), (q, want_q)):
                        err = (np.abs(got - want).max(-1) / np.abs(want).max(-1)).max()
                        assert err < 2e-2, (rho, b, err)
                xs[b] += g["tokens"]
                want_K = OH.candidate_length(list(s.astype(np.float64)) + [1.0] * 40, hh, k_max)
                if want_K != K:
                    ph = np.cumprod(np.concatenate([[1.0], s.astype(np.float64)]))
                    assert np.min(np.abs(1 - ph - hh)) < 1e-5
                    exempt += 1
                for i in range(1, K + 1):
                    qi = sampling.softmax(q[i - 1])
                    u = philox.uniform(seed, i, rho, b, philox.STREAM_DRAFT)
                    y = sampling.sample_inverse_cdf(qi, u)
                    assert y == g["cand"][i - 1] or sampling.cdf_margin(qi, u, y) < 1e-5, (rho, b, i)
                o = sampling.accept_resample(p, q, g["cand"], K, seed=seed, rnd=rho, seq=b)
                if o["n"] != g["n"]:
                    i = min(o["n"], g["n"]) + 1
                    assert abs(o["r"][i - 1] - o["ratio"][i - 1]) < 1e-3
                    o = sampling.accept_resample(p, q, g["cand"], K, seed=seed, rnd=rho, seq=b,
                                                 forced={("accept", i): 1 if g["n"] >= i else 0})
                    exempt += 1
                assert o["n"] == g["n"]
                assert o["token"] == g["tokens"][-1] or o["margin"] < 1e-5
                P[b] += g["n"] + 1
                st = ctx.sd_seq_state(b)
                assert st["P"] == P[b] and st["kv_len_target"] == P[b] - 1
        assert exempt <= max_exempt
        return seen_K
    finally:
        ctx.close()


def test_ragged_batch_of_eight_bf16_decision_replay():
    """Eight sequences (136 activation rows in the target pass when all draft K_max, ragged K per
    sequence otherwise, per-sequence rollback)."""
    seen_K = _ragged_batch_replay(8, 16, [0.8] * 4, seed=9, max_exempt=3)
    assert len(seen_K) > 1


def test_ragged_batch_through_the_row_stripe_kernels():
    """Three sequences on a pair 2048 wide: the draft steps carry 6 rows, the target passes 8 or fewer when the
    sequences stop early and more when they do not, so the rounds alternate between the row-stripe GEMM with its
    fused SiLU / residual / norm epilogues and the MFMA or tiled kernels with the separate small kernels, on the same
    caches; rows against the oracle's teacher-forced forward, decisions replayed."""
    seen_K = _ragged_batch_replay(3, 8, [0.3, 0.6, 0.9, 1.0, 0.5], seed=12, max_exempt=3, check_rows=3, wide=True)
    assert len(seen_K) > 1


def test_batch_at_the_row_limit():
    """Twenty sequences with K_max = 7: 20 x 8 = 160 target rows, the most a context takes, and 40
    draft rows per step (both through the tiled kernel); first every sequence drafts all 7 (h = 1),
    then the stop rule makes K ragged and the rows are packed."""
    seen_K = _ragged_batch_replay(20, 7, [1.0, 0.8, 0.8], seed=10, max_exempt=4, check_rows=4)
    assert 7 in seen_K and len(seen_K) > 1


@pytest.mark.parametrize("n_prompt", [1, 2, 3])
def test_very_short_prompts(n_prompt):
    """P = 1 means nothing to prefill (the first round ingests the only token); P = 2, 3
    exercise the first catch-up steps.  Greedy output must equal target-only greedy."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=11)
    prompt = synth.make_prompt(n_prompt, 1024, 40 + n_prompt)
    want = R.target_greedy_generate(oracle_model(t), prompt, 20)
    ctx = _context(t, d, h, k_max=4, max_seq=64)
    try:
        ctx.sd_prefill(0, prompt)
        seqs, st = ctx.specdec_generate(B.make_params(h=0.9, greedy=True), 20)
        assert seqs[0] == want
    finally:
        ctx.close()


def test_non_finite_logits_are_reported_and_cleared_by_prefill():
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=12)
    bad = dict(t)
    bad["lm_head"] = t["lm_head"].clone()
    bad["lm_head"][7, :] = float("inf")
    d2 = dict(d)
    d2["lm_head"] = bad["lm_head"]
    d2["tok_emb"] = bad["tok_emb"]
    d2["final_norm"] = bad["final_norm"]
    prompt = synth.make_prompt(8, 1024, 3)
    ctx = _context(bad, d2, h, k_max=4, max_seq=64)
    try:
        ctx.sd_prefill(0, prompt)
        with pytest.raises(B.SpecDecError) as e:
            ctx.specdec_round(B.make_params(h=0.7, seed=0))
        assert e.value.status == B.SD_ENONFINITE
        ctx.sd_prefill(0, prompt)              # clears the sticky flag; the weights are still bad
        with pytest.raises(B.SpecDecError) as e:
            ctx.specdec_round(B.make_params(h=0.7, seed=0))
        assert e.value.status == B.SD_ENONFINITE
    finally:
        ctx.close()


def test_eos_stops_generation_like_the_oracle():
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair(seed=13)
    prompt = synth.make_prompt(10, 1024, 6)
    tw, dw, hw = oracle_model(t), oracle_model(d), oracle_head(h)
    base, _, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=0.7, seed=2), 30, 6, 128, cached=True)
    eos = base[12]
    want, ost, _ = R.oracle_generate(tw, dw, hw, prompt, R.Params(h=0.7, seed=2, eos_id=eos), 30, 6, 128, cached=True)
    ctx = _context(t, d, h, k_max=6, max_seq=128)
    try:
        ctx.sd_prefill(0, prompt)
        seqs, st = ctx.specdec_generate(B.make_params(h=0.7, seed=2, eos_id=eos), 30)
        assert seqs[0] == want and want[-1] == eos and len(want) <= 13
        assert (st["N"], st["N_draft"], st["N_target"]) == (ost.N, ost.N_draft, ost.N_target)
    finally:
        ctx.close()


def test_first_emitted_token_of_a_round_follows_the_target():
    """Speculative sampling leaves the output distribution unchanged (Appendix C), whatever rule
    chose K: over 3000 seeds on the tiny pair, the first token a round emits (y_1 if accepted, else
    the residual draw) must be distributed as the target's p_1.  Tokens are binned into 16 groups
    of 64 consecutive ids; chi-square at the 99.9 % quantile of 15 degrees of freedom."""
    from paper_2405_19715_amd import binding as B
    from oracle.model import forward_full
    t, d, h = tiny_pair()
    prompt = synth.make_prompt(24, 1024, 11)
    p1 = sampling.softmax(forward_full(oracle_model(t), prompt)[0][-1])
    ctx = _context(t, d, h, k_max=8, max_seq=64)
    try:
        trials, bins = 3000, 16
        counts = np.zeros(bins)
        for seed in range(trials):
            ctx.sd_prefill(0, prompt)
            g = ctx.specdec_round(B.make_params(h=0.7, seed=1000 + seed))[0]
            counts[g["tokens"][0] * bins // 1024] += 1
        want = trials * p1.reshape(bins, -1).sum(-1)
        chi = ((counts - want) ** 2 / want).sum()
        assert want.min() > 50 and chi < 37.7, chi
    finally:
        ctx.close()


def test_rounds_on_a_stream_of_the_callers():
    """The context enqueues everything on the stream it was created with: built and driven under
    a non-default torch stream, the free-running token stream must match the oracle as on the
    default stream (a kernel or copy left on another stream would read data that is not there yet)."""
    from paper_2405_19715_amd import binding as B
    t, d, h = tiny_pair()
    prompt = synth.make_prompt(40, 1024, 21)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = _context(t, d, h, k_max=8, max_seq=192)
        try:
            ctx.sd_prefill(0, prompt)
            op = R.Params(h=0.7, temperature=1.0, greedy=False, seed=8)
            gp = B.make_params(h=0.7, temperature=1.0, greedy=False, seed=8)
            toks, exempt, hist = run_free_running(ctx, oracle_model(t), oracle_model(d), oracle_head(h), prompt, op, gp,
                                                  64, 8, 192)
            assert len(toks) == 64 and exempt <= 2
            # the isolated accept step on the same stream
            p, q = synth.make_accept_logits(2, 4, 1024, 3)
            cand = torch.zeros((2, 4), dtype=torch.int32)
            n, tok, flags = B.sd_accept_resample(p.cuda(), q.cuda(), cand.cuda(),
                                                 torch.full((2,), 4, dtype=torch.int32).cuda(), gp, 0)
            side.synchronize()
            for b in range(2):
                o = sampling.accept_resample(p[b].numpy(), q[b].numpy(), cand[b].numpy(), 4, seed=8, rnd=0, seq=b)
                assert int(n[b]) == o["n"]
        finally:
            ctx.close()
    side.synchronize()


def test_gemm_timers_rotate_over_the_layers_and_change_nothing():
    """sd_profile_enable(every) brackets the target pass's GEMM launches of every `every`-th layer, one layer
    further with each pass; sd_profile_read returns what piled up since the last read.  The counts and bytes
    are fixed by that rule, and the rounds must give the same tokens with the timers on."""
    from paper_2405_19715_amd import binding as B
    t, d, h = _bf16_pair()
    prompt = synth.make_prompt(40, 2048, 3)
    gp = B.make_params(h=0.8, temperature=1.0, greedy=False, seed=11)
    n_rounds, every = 7, 2
    runs = []
    for prof in (0, every):
        ctx = _context(t, d, h, k_max=8, max_seq=256)
        try:
            ctx.sd_prefill(0, prompt)
            ctx.sd_profile_enable(prof)
            ctx.sd_profile_read()
            out = []
            for _ in range(n_rounds):
                out += [(r["K"], r["n"], tuple(r["tokens"])) for r in ctx.specdec_round(gp)]
            stats = ctx.sd_profile_read()
            again = ctx.sd_profile_read()
            runs.append((out, stats, again))
        finally:
            ctx.close()
    (out0, st0, _), (out1, st1, again1) = runs
    assert out0 == out1
    assert all(v["launches"] == 0 for v in st0.values())
    assert all(v["launches"] == 0 and v["seconds"] == 0 for v in again1.values())      # a read empties the sums
    # two target layers, every = 2: pass p samples layer l with (l + p) % 2 == 0, i.e. exactly one layer per pass
    dm, nq, nkv, ffn, V = 512, 8 * 64, 1 * 64, 640, 2048          # the target of _bf16_pair()
    per = {"qkv": (nq + 2 * nkv) * dm, "o": dm * nq, "gate_up": 2 * ffn * dm, "down": dm * ffn, "lm_head": V * dm}
    for k, v in st1.items():
        assert v["launches"] == n_rounds, (k, v)
        assert v["weight_bytes"] == n_rounds * per[k] * 2
        assert 0 < v["seconds"] < 1.0
