"""CPU pins of tests/_bf16_rounding.py, the oracle's decoder with bf16 storage emulated: with the
rounding switched off it must BE the oracle's forward, whatever the chunking and launch modes; its
rounding function must be the library conversion; and with rounding on it must sit at bf16 distance
from the fp64 forward (a wrapper that rounded nothing, or too much, fails one of these)."""
import numpy as np
import torch

from oracle.model import forward_full
from paper_2405_19715_amd import synth
from tests._bf16_rounding import RoundedDecoder, bf16_round, identity
from tests._util import oracle_model


def _model(seed=3, layers=3, hq=4, hkv=2, std=0.3):
    shape = synth.ModelShape(layers, 64, hq, hkv, 16, 96, 50)
    return oracle_model(synth.make_model(shape, seed, dtype=torch.bfloat16, std=std))


def test_bf16_round_is_the_library_conversion():
    g = torch.Generator().manual_seed(0)
    a = torch.randn(20000, generator=g, dtype=torch.float32) * 3
    a[:4] = torch.tensor([0.0, -0.0, 1.00390625, 1.01171875])       # two exact ties between neighbours
    want = a.to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(bf16_round(a.numpy().astype(np.float64)), want)


def test_without_rounding_it_is_the_oracle_forward():
    w = _model()
    toks = synth.make_prompt(150, 50, 1)          # spans three 64-key blocks
    want = forward_full(w, toks)[0]
    for rows, fused, full in (((150,), (False,), (False,)), ((150,), (False,), (True,)),
                              ((100, 43, 7), (False, False, True), (True, False, False)),
                              ((64, 80, 6), (True, True, True), (False, True, False))):
        dec = RoundedDecoder(w, toks, rows, fused, full, rnd=identity)
        for i, lw in enumerate(w.layers):
            dec.layer(lw)
        s = 0
        for ci, r in enumerate(rows):
            got = dec.logits(ci)
            assert np.abs(got - want[s:s + r]).max() < 1e-9 * np.abs(want).max(), (rows, ci)
            s += r


def test_fp32_arithmetic_without_rounding_is_the_oracle_forward_to_fp32_accuracy():
    w = _model(std=0.1)
    toks = synth.make_prompt(70, 50, 1)
    want = forward_full(w, toks)[0][-6:]
    dec = RoundedDecoder(w, toks, (64, 6), (False, True), (True, False), rnd=identity, dtype=np.float32)
    for lw in w.layers:
        dec.layer(lw)
    got = dec.logits()
    assert got.dtype == np.float64 and dec.chunks[-1].x.dtype == np.float32
    err = np.abs(got - want).max() / np.abs(want).max()
    assert 1e-9 < err < 1e-5, err


def test_with_rounding_it_sits_at_bf16_distance():
    w = _model(seed=5, std=0.1)
    toks = synth.make_prompt(90, 50, 2)
    want = forward_full(w, toks)[0][-6:]
    errs = []
    for fused in (False, True):
        dec = RoundedDecoder(w, toks, (84, 6), (False, fused), (True, False))
        for lw in w.layers:
            dec.layer(lw)
        got = dec.logits()
        errs.append((np.abs(got - want).max(-1) / np.abs(want).max(-1)).max())
    # bf16 keeps 8 bits: a handful of roundings per layer give an error of order 2^-9 .. 2^-6
    assert all(2.0 ** -12 < e < 2.0 ** -5 for e in errs), errs
    assert errs[0] != errs[1]                    # deferring the row factor moves a rounding point
