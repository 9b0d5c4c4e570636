"""Parity of the head-training path (Sec. 4.4: training-set construction with token mixing,
weighted BCE, gradients, Adam) with the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import train as OT
from oracle.head import HeadWeights
from paper_2405_19715_amd import synth
from tests._util import oracle_head, oracle_model
from tests.test_gpu_round import _bf16_pair, _context, tiny_pair

pytestmark = pytest.mark.gpu


def test_examples_match_oracle_on_the_tiny_pair():
    t, d, h = tiny_pair(seed=2)
    prompt = synth.make_prompt(20, 1024, 5)
    X = synth.make_prompt(45, 1024, 6)             # any token sequence serves as the response here
    ctx = _context(t, d, h, k_max=8, max_seq=128)
    try:
        for top_k in (0, 20):
            E, P, mask, Y, Z = ctx.sd_head_examples(0, prompt, X, r=0.15, seed=11, example=3, temperature=0.9,
                                                    top_k=top_k)
            wE, wP, wmask, wY, wZ = OT.make_examples(oracle_model(t), oracle_model(d), prompt, X, 0.15, 11, 3,
                                                     temperature=0.9, top_k=top_k)
            assert Y == [int(v) for v in wY] and Z == [int(v) for v in wZ]
            assert mask.cpu().tolist() == [int(v) for v in wmask]
            np.testing.assert_allclose(P.cpu().numpy(), wP, rtol=0, atol=2e-3)
            got = E.cpu().numpy()
            err = np.abs(got - wE).max(-1) / np.abs(wE).max(-1)
            assert err.max() < 1e-4
        # the slot has to be prefilled again before it decodes
        from paper_2405_19715_amd import binding as B
        with pytest.raises(B.SpecDecError):
            ctx.specdec_round(B.make_params())
        ctx.sd_prefill(0, prompt)
        assert ctx.specdec_round(B.make_params(seed=1))[0]["K"] >= 1
    finally:
        ctx.close()


def test_examples_on_a_bf16_pair_are_consistent_with_the_forward_pass():
    t, d, h = _bf16_pair()
    prompt = synth.make_prompt(33, 2048, 1)
    X = synth.make_prompt(70, 2048, 2)
    ctx = _context(t, d, h, k_max=8, max_seq=256)
    try:
        E, P, mask, Y, Z = ctx.sd_head_examples(0, prompt, X, r=0.3, seed=4, example=0)
        P, mask = P.cpu().numpy(), mask.cpu().numpy()
        assert ((P >= 0) & (P <= 1)).all() and 0.0 < P.mean() < 1.0
        for i in range(70):
            assert Z[i] == (Y[i] if mask[i] else X[i])
        assert 5 <= (mask == 0).sum() <= 40
        # E_i is the draft's final embedding of Z_i given (prompt, Z_<i): the teacher-forced forward gives it too
        ctx.sd_prefill(0, prompt)
        toks = prompt[-1:] + Z
        rows = []
        for s0 in range(0, 71, 32):
            _, hid = ctx.sd_forward(1, 0, 32 + s0, toks[s0:s0 + 32], want_hidden=True)
            rows.append(hid.numpy())
        np.testing.assert_array_equal(np.concatenate(rows)[1:], E.cpu().numpy())
        # and the oracle's forward over the same mixed sequence agrees to the bf16 tolerance
        wE, wP, *_ = OT.make_examples(oracle_model(t), oracle_model(d), prompt, X, 0.3, 4, 0)
        from oracle.model import forward_full
        _, hid = forward_full(oracle_model(d), prompt + Z)
        want = hid[33:33 + 70]
        assert (np.abs(E.cpu().numpy() - want).max(-1) / np.abs(want).max(-1)).max() < 2e-2
    finally:
        ctx.close()


def _rand_head(dims, residual, seed):
    h = synth.make_head(dims, seed, dtype=torch.float32, residual=residual, std=0.2, out_bias=0.5)
    g = torch.Generator().manual_seed(seed + 1)
    h["b"] = [b + 0.1 * torch.randn(b.shape, generator=g) for b in h["b"]]
    return h


def _cuda_head(h):
    out = dict(h)
    out["W"] = [w.cuda() for w in h["W"]]
    out["b"] = [b.cuda() for b in h["b"]]
    return out


def _batch(n, d, seed):
    g = torch.Generator().manual_seed(seed)
    E = torch.randn((n, d), generator=g)
    P = torch.rand((n,), generator=g)
    mask = (torch.rand((n,), generator=g) < 0.8).to(torch.int32)
    return E, P, mask


@pytest.mark.parametrize("dims,residual,n", [([64, 64, 64, 1], True, 37), ([48, 80, 32, 1], False, 130),
                                             ([100, 1], False, 5), ([256, 256, 256, 256, 256, 1], True, 300)])
def test_loss_and_gradients_match_oracle(dims, residual, n):
    from paper_2405_19715_amd import binding as B
    h = _rand_head(dims, residual, 3)
    E, P, mask = _batch(n, dims[0], 4)
    want_loss, gW, gb = OT.head_loss_grad(oracle_head(h), E.double().numpy(), P.double().numpy(), mask.numpy(),
                                          w_acc=1.0, w_rej=6.0)
    tr = B.Trainer(_cuda_head(h), n_max=512)
    try:
        loss = tr.sd_trainer_step(E.cuda(), P.cuda(), mask.cuda(), w_acc=1.0, w_rej=6.0, apply=False)
        assert abs(loss - want_loss) < 1e-5 * max(1.0, abs(want_loss))
        for j in range(len(dims) - 1):
            for what, want in ((2, gW[j]), (3, gb[j])):
                got = tr.sd_trainer_read(j, what).double().numpy().reshape(want.shape)
                assert np.abs(got - want).max() < 2e-5 * max(np.abs(want).max(), 1e-3), (j, what)
            # apply = False left the weights alone
            np.testing.assert_array_equal(tr.sd_trainer_read(j, 0).numpy(), h["W"][j].numpy())
        lg = tr.sd_trainer_predict(E.cuda()).cpu().double().numpy()
        want_lg, _, _ = OT.head_forward_batch(oracle_head(h), E.double().numpy())
        np.testing.assert_allclose(lg, want_lg, rtol=0, atol=2e-5 * max(1.0, np.abs(want_lg).max()))
    finally:
        tr.close()


def test_adam_trajectory_matches_oracle_and_export_round_trips():
    from paper_2405_19715_amd import binding as B
    dims = [32, 32, 32, 1]
    h = _rand_head(dims, True, 7)
    oh = oracle_head(h)
    oh = HeadWeights(W=[w.copy() for w in oh.W], b=[b.copy() for b in oh.b], residual=True)
    batches = [_batch(64, 32, 100 + s) for s in range(12)]
    want_losses = OT.train_steps(oh, [(E.double().numpy(), P.double().numpy(), m.numpy()) for E, P, m in batches],
                                 w_acc=1.0, w_rej=3.0, lr=1e-2)
    tr = B.Trainer(_cuda_head(h), n_max=64)
    try:
        losses = [tr.sd_trainer_step(E.cuda(), P.cuda(), m.cuda(), w_acc=1.0, w_rej=3.0, lr=1e-2)
                  for E, P, m in batches]
        np.testing.assert_allclose(losses, want_losses, rtol=2e-4)
        assert losses[-1] < losses[0]
        for j in range(3):
            for what, want in ((0, oh.W[j]), (1, oh.b[j])):
                got = tr.sd_trainer_read(j, what).double().numpy().reshape(want.shape)
                diff = np.sort(np.abs(got - want).ravel())
                # Adam divides by sqrt(v): an entry whose gradient is at rounding level may move
                # the other way in fp32, so a handful of entries are allowed one step's worth
                assert diff[int(0.99 * (len(diff) - 1))] < 2e-4 and diff[-1] < 12 * 1e-2
        exp = tr.sd_trainer_export(torch.bfloat16)
        for j in range(3):
            np.testing.assert_array_equal(exp["W"][j].cpu().float().numpy(),
                                          tr.sd_trainer_read(j, 0).to(torch.bfloat16).float().numpy())
        assert exp["dims"] == dims and exp["residual"]
    finally:
        tr.close()


def test_trainer_rejects_bad_arguments():
    from paper_2405_19715_amd import binding as B
    h = _rand_head([16, 1], False, 1)
    tr = B.Trainer(_cuda_head(h), n_max=8)
    try:
        E, P, m = _batch(9, 16, 1)
        with pytest.raises(B.SpecDecError):
            tr.sd_trainer_step(E.cuda(), P.cuda(), m.cuda())          # more rows than n_max
        E, P, m = _batch(4, 16, 1)
        with pytest.raises(B.SpecDecError):
            tr.sd_trainer_step(E.cuda(), P.cuda(), m.cuda(), beta1=1.0)
    finally:
        tr.close()


def test_training_learns_a_learnable_target():
    """Targets that are a logistic function of the embedding are recovered by a D = 1 head:
    the held-out prediction correlates with the target (the synthetic model pairs give
    targets that do not depend on the embedding, so this is the check that the trainer
    learns when there is something to learn)."""
    from paper_2405_19715_amd import binding as B
    g = torch.Generator().manual_seed(0)
    d = 64
    w_true = torch.randn(d, generator=g)
    h = synth.make_head([d, d, 1], 5, dtype=torch.float32, residual=True, std=0.05, out_bias=0.0)
    tr = B.Trainer(_cuda_head(h), n_max=256)
    try:
        first = last = None
        for step in range(400):
            E = torch.randn((256, d), generator=g)
            P = torch.sigmoid(E @ w_true / 4.0)
            last = tr.sd_trainer_step(E.cuda(), P.cuda(), torch.ones(256, dtype=torch.int32).cuda(), lr=3e-3)
            first = first if first is not None else last
        E = torch.randn((256, d), generator=g)
        P = torch.sigmoid(E @ w_true / 4.0)
        pred = torch.sigmoid(tr.sd_trainer_predict(E.cuda()).cpu())
        assert last < first - 0.02
        assert float(torch.corrcoef(torch.stack([pred, P]))[0, 1]) > 0.97
    finally:
        tr.close()
