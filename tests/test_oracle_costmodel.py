"""Pins for oracle/costmodel.py: the arithmetic on the numbers the paper prints
(Sec. 5.2, Table 1, Sec. 1, Sec. 4.1) and the identity behind Lemma 1."""
import os

import numpy as np

from oracle import costmodel as C

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_throughput.txt")


def _paper():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_target_only_throughput():
    p = _paper()
    assert round(C.target_only_tokens_per_second(p["t_target_standalone"]), 2) == p["target_only_tps"]


def test_speedups_are_throughput_ratios():
    p = _paper()
    for ds in ("alpaca", "humaneval", "gsm8k"):
        for algo in ("specdecpp", "specdec"):
            assert round(p[f"{algo}_tps_{ds}"] / p["target_only_tps"], 2) == p[f"{algo}_speedup_{ds}"]
    assert round(p["oracle_tps"] / p["target_only_tps"], 2) == p["oracle_speedup"]


def test_hindsight_oracle_throughput_from_eq4():
    """Sec. 4.1: no discards and N_target/N = 0.164 at the speculative-setting
    forward times gives about the printed 27.06 tokens/s (the paper averages
    per-prompt throughputs, so only approximately)."""
    p = _paper()
    tps = C.tokens_per_second(p["t_draft"], p["t_target"], 0.0, p["oracle_verification_rate"])
    assert abs(tps - p["oracle_tps"]) / p["oracle_tps"] < 0.05


def test_eq1_equals_lemma1_when_counter_identity_holds():
    rng = np.random.default_rng(0)
    for _ in range(100):
        n_target = int(rng.integers(1, 50))
        n_draft = int(rng.integers(n_target, 20 * n_target))
        n_disc = int(rng.integers(0, n_draft))
        n = n_draft + n_target - n_disc
        td, tt = rng.uniform(0.001, 0.05), rng.uniform(0.05, 0.2)
        t1 = C.total_time(td, tt, n_draft, n_target)
        t2 = C.total_time_decomposed(td, tt, n, n_disc, n_target)
        assert abs(t1 - t2) < 1e-12
        assert abs(C.latency_per_token(td, tt, n_disc / n, n_target / n) - t1 / n) < 1e-12
