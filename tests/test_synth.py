"""The seeded input generators: the recipes that give a synthetic pair a chosen degree of
agreement are checked against what their construction predicts, with the oracle's forward."""
from math import erf, sqrt

import numpy as np
import pytest
import torch

from oracle.model import forward_full
from oracle.sampling import softmax
from paper_2405_19715_amd import synth
from tests._util import oracle_model


@pytest.mark.parametrize("extra_gain", [1.0, 2.0])
def test_aligned_pair_of_different_widths_has_the_predicted_acceptance(extra_gain):
    """align_narrow_draft: the draft sees the first d_draft columns of the target's logit sum, the
    rest is a per-token shift of standard deviation sigma = 0.02 * extra_gain * sqrt(d_target -
    d_draft); for a log-normal ratio the acceptance sum_v min(p_v, q_v) is 2 Phi(-sigma / 2)."""
    ts = synth.ModelShape(2, 1024, 8, 2, 128, 1536, 4096)
    ds = synth.ModelShape(1, 512, 4, 4, 128, 768, 4096)
    t = synth.make_model(ts, 1, dtype=torch.float32)
    d = synth.make_model(ds, 2, dtype=torch.float32)
    synth.align_narrow_draft(t, d, 1e-4, extra_gain)
    toks = synth.make_prompt(24, 4096, 3)
    p = softmax(forward_full(oracle_model(t), toks)[0])
    q = softmax(forward_full(oracle_model(d), toks)[0])
    alpha = np.minimum(p, q).sum(-1)
    sigma = 0.02 * extra_gain * sqrt(1024 - 512)
    want = 1 + erf(-sigma / 2 / sqrt(2))                   # 2 Phi(-sigma / 2)
    assert abs(alpha.mean() - want) < 0.02 and alpha.min() > want - 0.05
    # an independent random draft of the same shape agrees much less
    r = synth.make_model(ds, 5, dtype=torch.float32)
    synth.damp_tail(r, 0, 1e-4)
    qr = softmax(forward_full(oracle_model(r), toks)[0])
    assert np.minimum(p, qr).sum(-1).mean() < alpha.mean() - 0.05
