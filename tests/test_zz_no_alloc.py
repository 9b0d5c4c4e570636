"""The entry point that allocates nothing (sd_accept_resample_static: row statistics in a device
array of the library image) against sd_accept_resample with a caller's workspace: same inputs,
bit-equal outputs, on two calls in a row, the second with a smaller input, so that whatever the
first call left in the shared array would show.  Collected last: it shares no state with the
other tests, but a failure here must not hide them."""
import numpy as np
import pytest
import torch

from oracle import philox, sampling
from paper_2405_19715_amd import synth

pytestmark = pytest.mark.gpu


def _case(B, Kmax, V, seed, greedy, top_k):
    p, q = synth.make_accept_logits(B, Kmax, V, seed)
    rng = np.random.default_rng(seed)
    Ks = rng.integers(0, Kmax + 1, size=B).astype(np.int32)
    cand = np.zeros((B, Kmax), dtype=np.int32)
    for b in range(B):
        if greedy:
            cand[b, : Ks[b]] = q[b, : Ks[b]].argmax(-1).numpy()
        else:
            qq = sampling.softmax(sampling.warp_top_k(q[b, : Ks[b]].double().numpy(), top_k)) if Ks[b] else []
            cand[b, : Ks[b]] = [sampling.sample_inverse_cdf(qq[i], philox.uniform(seed, i + 1, 3, b, philox.STREAM_DRAFT))
                                for i in range(Ks[b])]
    return p.cuda(), q.cuda(), torch.from_numpy(cand).cuda(), torch.from_numpy(Ks).cuda()


def test_static_scratch_entry_point_equals_the_workspace_one():
    from paper_2405_19715_amd import binding as Bd
    dev = "cuda"
    # first call large (the array's full batch), second smaller in every dimension
    for (B, Kmax, V, seed, greedy, top_k) in ((64, 16, 32000, 5, False, 0), (3, 4, 1000, 6, False, 50),
                                             (7, 8, 32000, 7, True, 0)):
        p, q, cand, Ks = _case(B, Kmax, V, seed, greedy, top_k)
        params = Bd.make_params(seed=seed, greedy=greedy, top_k=top_k)
        want = Bd.sd_accept_resample(p, q, cand, Ks, params, 3)
        out = (torch.full((B,), -7, dtype=torch.int32, device=dev), torch.full((B,), -7, dtype=torch.int32, device=dev),
               torch.full((B, Kmax), 9, dtype=torch.uint8, device=dev))
        before = torch.cuda.memory_allocated()
        word = Bd.sd_accept_resample_static(p, q, cand, Ks, params, 3, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert word
        for g, w in zip(out, want):
            assert torch.equal(g, w)
        # and against the oracle, sequence by sequence (the workspace entry's own bar)
        n, tok, flags = (o.cpu().numpy() for o in out)
        for b in range(0, B, max(1, B // 4)):
            o = sampling.accept_resample(p[b].cpu().numpy(), q[b].cpu().numpy(), cand[b].cpu().numpy(), int(Ks[b]),
                                         greedy=greedy, seed=seed, rnd=3, seq=b, top_k=top_k)
            if (flags[b, : Ks[b]] == o["flags"]).all():
                assert n[b] == o["n"] and (tok[b] == o["token"] or (not greedy and o["margin"] < 1e-5))
            else:
                i = int(np.argmax(flags[b, : Ks[b]] != o["flags"]))
                assert abs(o["r"][i] - o["ratio"][i]) < 1e-3


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    from paper_2405_19715_amd import binding as Bd
    B, Kmax, V = Bd.lib_static_max_batch() + 1, 2, 64
    p = torch.zeros((B, Kmax + 1, V), device="cuda")
    q = torch.zeros((B, Kmax, V), device="cuda")
    cand = torch.zeros((B, Kmax), dtype=torch.int32, device="cuda")
    Ks = torch.zeros((B,), dtype=torch.int32, device="cuda")
    out = (torch.zeros(B, dtype=torch.int32, device="cuda"), torch.zeros(B, dtype=torch.int32, device="cuda"),
           torch.zeros((B, Kmax), dtype=torch.uint8, device="cuda"))
    with pytest.raises(Bd.SpecDecError) as e:
        Bd.sd_accept_resample_static(p, q, cand, Ks, Bd.make_params(), 0, out)
    assert e.value.status == Bd.SD_ERANGE
