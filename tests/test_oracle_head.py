"""Pins for oracle/head.py: brute-force search of the stop index (chain rule of
Sec. 4.3), closed-form special cases, and the head MLP against torch's own
Linear / SiLU / sigmoid routines."""
import itertools
from fractions import Fraction

import numpy as np
import torch

from oracle import head as H


def _brute_force_K(s, h, k_cap):
    """Smallest i >= 1 such that 1 - prod_{j < i} s_j > h, each product recomputed
    from scratch; k_cap if there is none."""
    for i in range(1, k_cap + 1):
        prod = Fraction(1)
        for j in range(i - 1):
            prod *= Fraction(s[j])
        if 1 - prod > Fraction(h):
            return i
    return k_cap


def test_stop_index_brute_force():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        k_cap = int(rng.integers(1, 10))
        s = rng.uniform(0.3, 1.0, size=k_cap).tolist()
        h = float(rng.choice([0.1, 0.3, 0.5, 0.7, 0.9, rng.uniform(0, 1)]))
        want = _brute_force_K(s, h, k_cap)
        got = H.candidate_length(s, h, k_cap)
        if got != want:
            # only a product within rounding of the threshold may differ
            prod = np.prod(s[: min(got, want) - 1 + 1])
            assert abs(1 - prod - h) < 1e-12
        else:
            assert got == want


def test_stop_rule_special_cases():
    s = [0.8] * 32
    assert H.candidate_length(s, 1.0, 16) == 16          # h >= 1: fixed K (Algorithm 1)
    assert H.candidate_length(s, 1.5, 7) == 7
    assert H.candidate_length(s, -0.1, 16) == 1          # h < 0: stop at once
    assert H.candidate_length([1.0] * 32, 0.5, 16) == 16  # certain acceptance never stops
    # constant s = 0.8: smallest i with 1 - 0.8^(i-1) > h
    for h, want in [(0.3, 3), (0.5, 5), (0.7, 7), (0.9, 12)]:
        assert H.candidate_length(s, h, 20) == want
    # the comparison is strict
    assert H.should_stop(0.5, 0.5) is False or H.should_stop(0.5, 0.5) == False  # noqa: E712
    assert H.should_stop(0.49, 0.5)


def test_all_binary_head_outputs_small_case():
    """Every 0/1-valued prediction pattern of length 4: the round stops one draw
    after the first predicted rejection (h in [0,1))."""
    for pattern in itertools.product([0.0, 1.0], repeat=4):
        first_zero = next((i for i, v in enumerate(pattern) if v == 0.0), None)
        want = 5 if first_zero is None else first_zero + 2
        assert H.candidate_length(list(pattern), 0.5, 5) == min(want, 5)


def _torch_head(dims, residual, seed):
    g = torch.Generator().manual_seed(seed)
    lins = []
    for j in range(len(dims) - 1):
        lin = torch.nn.Linear(dims[j], dims[j + 1]).double()
        with torch.no_grad():
            lin.weight.copy_(torch.randn(lin.weight.shape, generator=g, dtype=torch.float64) * 0.3)
            lin.bias.copy_(torch.randn(lin.bias.shape, generator=g, dtype=torch.float64) * 0.3)
        lins.append(lin)

    def f(e):
        z = torch.as_tensor(e, dtype=torch.float64)
        for lin in lins[:-1]:
            a = torch.nn.functional.silu(lin(z))
            z = z + a if (residual and lin.in_features == lin.out_features) else a
        return torch.sigmoid(lins[-1](z)).item()

    hw = H.HeadWeights(W=[l.weight.detach().numpy() for l in lins],
                       b=[l.bias.detach().numpy() for l in lins], residual=residual)
    return f, hw


def test_head_matches_torch_modules():
    rng = np.random.default_rng(1)
    for dims, residual in [([16, 1], False), ([16, 8, 1], False), ([12, 12, 12, 12, 1], True),
                           ([12, 12, 12, 12, 1], False), ([10, 6, 6, 1], True)]:
        f, hw = _torch_head(dims, residual, seed=len(dims))
        for _ in range(5):
            e = rng.normal(size=dims[0])
            assert abs(H.accept_prob(hw, e) - f(e)) < 1e-13


def test_sigmoid_is_scipy_expit():
    from scipy.special import expit
    for z in [-800.0, -30.0, -1.0, 0.0, 1.386, 40.0, 800.0]:
        assert abs(H.sigmoid(z) - expit(z)) < 1e-15
    assert abs(H.sigmoid(1.386) - 0.8) < 1e-3
