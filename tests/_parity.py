"""Free-running parity harness: the HIP path and the oracle decode independently
from the same seed; streams must agree decision by decision.  Where they differ the
oracle's own margin at that decision must be inside the stated tolerance (a
near-tie the two precisions may break differently); the oracle is then pushed
through the HIP path's decision and the comparison continues."""
from oracle import rounds as R

TOL = {"accept": 1e-3, "draft": 1e-5, "token": 1e-5, "stop": 1e-5, "greedy": 1e-5}


def _trace_margin(trace, kind, i):
    for k, ii, _, margin in trace:
        if k == kind and ii == i:
            return margin
    raise KeyError((kind, i))


def _first_mismatch(g, o):
    """(forced-key, forced-value, kind, margin) of the first decision where the HIP
    round g and the oracle round o part ways, or None."""
    for i in range(1, min(g["K"], o["K"]) + 1):
        if g["cand"][i - 1] != o["cand"][i - 1]:
            return ("draft", i), g["cand"][i - 1], "draft", _trace_margin(o["trace"], "draft", i)
    if g["K"] != o["K"]:
        i = min(g["K"], o["K"])
        return ("stop", i), g["K"] == i, "stop", _trace_margin(o["trace"], "stop", i)
    if g["n"] != o["n"]:
        i = min(g["n"], o["n"]) + 1
        return ("accept", i), 1 if g["n"] >= i else 0, "accept", _trace_margin(o["trace"], "accept", i)
    if g["tokens"][-1] != o["tokens"][-1]:
        return "token", g["tokens"][-1], "token", _trace_margin(o["trace"], "token", o["n"] + 1)
    return None


def run_free_running(ctx, tw, dw, hw, prompt, oparams, gparams, max_new, k_max, max_seq, seq=0):
    """Returns (tokens, exempt events, per-round (K, n)).  Raises AssertionError on a
    mismatch outside the tolerances."""
    target, draft = R.Cached(tw), R.Cached(dw)
    x = [int(t) for t in prompt]
    out, exempt, hist, rho = [], 0, [], 0
    while len(out) < max_new:
        g = ctx.specdec_round(gparams)[seq]
        forced = {}
        while True:
            o = R.oracle_round(target, draft, hw, x, rho, oparams, k_max, max_seq, seq, forced)
            mm = _first_mismatch(g, o)
            if mm is None:
                break
            key, val, kind, margin = mm
            tol = TOL["greedy"] if oparams.greedy and kind in ("draft", "accept", "token") else TOL[kind]
            assert key not in forced, f"round {rho}: forcing {key} did not reconcile the streams"
            assert margin < tol, f"round {rho}: {kind} decision {key} differs, oracle margin {margin:.3e} >= {tol}"
            forced[key] = val
            exempt += 1
        assert g["tokens"] == o["tokens"] and g["K"] == o["K"] and g["n"] == o["n"]
        x += o["tokens"]
        out += o["tokens"]
        hist.append((o["K"], o["n"]))
        rho += 1
    return out[:max_new], exempt, hist
