"""Condense a `rocprofv3 --kernel-trace --output-format csv` trace of bench.py into a
short text summary per phase of a round.

    python -m paper_2405_19715_amd.profile_summary <..._kernel_trace.csv> [--skip-rounds W]
    python -m paper_2405_19715_amd.profile_summary <..._counter_collection.csv> --pmc | --counters
    python -m paper_2405_19715_amd.profile_summary <..._kernel_trace.csv> --by-grid accept_k,row_stats_k

The whole-process statistics rocprofv3 prints mix the untimed prefill (which runs the
same GEMM kernel over 32-row prompt chunks of both models) into every average.  This
script cuts the trace at the kernels that open a round (begin_round_k) and a target
pass (plan_verify_k) and reports the rounds after the first `--skip-rounds` only.
"""
from __future__ import annotations

import argparse
import collections
import csv
import re
import sys


STREAMING = ("gemm_bf16_str", "gemm_bf16_mstripe")     # gemm_bf16_stripe<M>, gemm_bf16_stream<NT>, gemm_bf16_mstripe<..>


def is_streaming(name: str) -> bool:
    return any(s in name for s in STREAMING)


def short_name(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "")
    m = re.match(r"(?:void )?([\w:]+(?:<[^(]*>)?)", name)
    return (m.group(1) if m else name)[:48]


def load(path):
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((short_name(r["Kernel_Name"]), int(r["Start_Timestamp"]), int(r["End_Timestamp"])))
    rows.sort(key=lambda r: r[1])
    return rows


def table(segments, title, out):
    """segments: list of launch lists, each one contiguous stretch of the stream."""
    agg = collections.OrderedDict()
    for rows in segments:
        for name, s, e in rows:
            a = agg.setdefault(name, [0, 0])
            a[0] += 1
            a[1] += e - s
    busy = sum(a[1] for a in agg.values())
    span = sum(rows[-1][2] - rows[0][1] for rows in segments)
    out.write(f"{title}: {sum(len(r) for r in segments)} launches, busy {busy / 1e6:.3f} ms, span {span / 1e6:.3f} ms, "
              f"idle between kernels {(span - busy) / 1e6:.3f} ms\n")
    for name, (n, t) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        out.write(f"  {name:48s} calls {n:6d}  avg {t / n / 1e3:9.2f} us  total {t / 1e6:9.3f} ms  {100.0 * t / span:5.1f}%\n")
    # the weight-streaming GEMMs come as several kernels (one stripe instantiation per row count, the MFMA kernel)
    ws = [(n, t) for name, (n, t) in agg.items() if is_streaming(name)]
    if len(ws) > 1:
        n, t = sum(a for a, _ in ws), sum(b for _, b in ws)
        out.write(f"  {'all weight-streaming GEMMs (stripe / mstripe / stream)':48s} calls {n:6d}  avg {t / n / 1e3:9.2f} us  "
                  f"total {t / 1e6:9.3f} ms  {100.0 * t / span:5.1f}%\n")


def pmc_summary(path, skip_rounds, out):
    """Per-launch HBM traffic of the target pass's GEMM kernel from a
    `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv` run of
    `bench.py --calibrate-copy`: the counter (KiB) is scaled by what it reads for the
    1 GiB device-to-device copies bench.py issues first."""
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Dispatch_Id"]), short_name(r["Kernel_Name"]), r["Counter_Name"], float(r["Counter_Value"])))
    rows.sort()
    counter = rows[0][2]
    copies = sorted(v for _, n, _, v in rows if "copyBuffer" in n)[-4:]
    scale = (1 << 20) / (sum(copies) / len(copies))          # KiB moved per counter unit
    out.write(f"counter {counter}: the 1 GiB copies read {sum(copies) / len(copies):.1f} per launch -> "
              f"{scale:.4f} KiB per counter unit\n")
    starts = [i for i, r in enumerate(rows) if "begin_round_k" in r[1]][skip_rounds:]
    per_grid = collections.OrderedDict()
    n_pass = 0
    for a, b in zip(starts, starts[1:] + [len(rows)]):
        rnd = rows[a:b]
        cut = next((i for i, r in enumerate(rnd) if "plan_verify" in r[1]), None)
        end = next((i for i, r in enumerate(rnd) if "commit_k" in r[1]), None)
        if cut is None or end is None:
            continue
        n_pass += 1
        for _, n, _, v in rnd[cut:end]:
            if is_streaming(n):
                a2 = per_grid.setdefault("gemm_bf16_stripe<*> + gemm_bf16_mstripe<*> + gemm_bf16_stream<*> (target pass)", [0, 0.0])
                a2[0] += 1
                a2[1] += v
    for k, (n, tot) in per_grid.items():
        out.write(f"{k}: {n} launches in {n_pass} target passes, {counter} per launch "
                  f"{tot / n * scale * 1024 / 1e6:.2f} MB (scaled), per pass {tot / n_pass * scale * 1024 / 1e9:.3f} GB\n")


def counters_summary(path, skip_rounds, out):
    """Per-launch averages of every counter in a `rocprofv3 --pmc <counters> --output-format csv`
    run of bench.py, for the GEMM launches of the target passes (everything between the kernel that
    plans the verify rows and the round's end)."""
    rows = []
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Dispatch_Id"]), short_name(r["Kernel_Name"]), r["Counter_Name"], float(r["Counter_Value"])))
    rows.sort()
    starts = [i for i, r in enumerate(rows) if "begin_round_k" in r[1]]
    starts = sorted(set(starts))
    # one row per (dispatch, counter): a round opens at the first row of a begin_round_k dispatch
    first = {}
    for i in starts:
        first.setdefault(rows[i][0], i)
    starts = sorted(first.values())[skip_rounds:]
    agg = collections.OrderedDict()
    for a, b in zip(starts, starts[1:] + [len(rows)]):
        rnd = rows[a:b]
        cut = next((i for i, r in enumerate(rnd) if "plan_verify" in r[1]), None)
        end = next((i for i, r in enumerate(rnd) if "commit_k" in r[1]), None)
        if cut is None or end is None:
            continue
        for d, n, c, v in rnd[cut:end]:
            if "gemm_bf16" in n:
                e = agg.setdefault((n, c), [set(), 0.0])
                e[0].add(d)
                e[1] += v
    for (n, c), (ds, tot) in agg.items():
        out.write(f"{n:40s} {c:36s} {tot / len(ds):18.1f} per launch ({len(ds)} launches)\n")


def by_grid(path, patterns, out):
    """Average duration per (kernel, grid in workgroups) of the kernels whose name holds one of
    `patterns`: for benchmarks that run one kernel over several problem sizes."""
    agg = collections.OrderedDict()
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            name = short_name(r["Kernel_Name"])
            if not any(p in name for p in patterns):
                continue
            wx, wy = max(int(r.get("Workgroup_Size_X", 1) or 1), 1), max(int(r.get("Workgroup_Size_Y", 1) or 1), 1)
            key = (name.replace("sd::", ""), int(r["Grid_Size_X"]) // wx, int(r.get("Grid_Size_Y", 1) or 1) // wy)
            a = agg.setdefault(key, [0, 0])
            a[0] += 1
            a[1] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    for (name, gx, gy), (n, t) in sorted(agg.items()):
        out.write(f"{name:28s} grid ({gx:3d}, {gy:3d})  calls {n:4d}  avg {t / n / 1e3:8.2f} us\n")


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("trace")
    ap.add_argument("--skip-rounds", type=int, default=2)
    ap.add_argument("--pmc", action="store_true", help="the file is a counter_collection.csv of a --pmc run")
    ap.add_argument("--counters", action="store_true",
                    help="the file is a counter_collection.csv: average every counter over the target pass's GEMM launches")
    ap.add_argument("--by-grid", default="", metavar="NAMES",
                    help="comma-separated kernel name fragments: average duration per (kernel, grid) instead of per round")
    args = ap.parse_args(argv)
    if args.by_grid:
        by_grid(args.trace, [p for p in args.by_grid.split(",") if p], sys.stdout)
        return
    if args.pmc:
        pmc_summary(args.trace, args.skip_rounds, sys.stdout)
        return
    if args.counters:
        counters_summary(args.trace, args.skip_rounds, sys.stdout)
        return
    rows = load(args.trace)
    starts = [i for i, r in enumerate(rows) if "begin_round_k" in r[0]]
    if len(starts) <= args.skip_rounds:
        raise SystemExit("trace holds too few rounds")
    first_round = starts[0]
    starts = starts[args.skip_rounds:]
    draft, verify = [], []
    n_rounds = 0
    for a, b in zip(starts, starts[1:] + [len(rows)]):
        rnd = rows[a:b]
        cut = next((i for i, r in enumerate(rnd) if "plan_verify" in r[0]), None)
        commit = next((i for i, r in enumerate(rnd) if "commit_k" in r[0]), None)
        if cut is None or commit is None:
            continue
        draft.append(rnd[:cut])
        verify.append(rnd[cut:commit + 1])
        n_rounds += 1
    out = sys.stdout
    out.write(f"rounds summarised: {n_rounds} (first {args.skip_rounds} skipped)\n")
    d_steps = sum(sum(1 for r in d if "plan_draft_k" in r[0]) for d in draft)
    d_span = sum(d[-1][2] - d[0][1] for d in draft)
    v_span = sum(v[-1][2] - v[0][1] for v in verify)
    out.write(f"draft steps: {d_steps}, mean draft-step span {d_span / max(d_steps, 1) / 1e6:.3f} ms; "
              f"mean target pass + accept span {v_span / n_rounds / 1e6:.3f} ms\n")
    prompt = [r for r in rows[:first_round] if r[0].startswith("sd::")]
    if prompt:
        table([prompt], "prompt pass of both models (before the first round, warm-up call included)", out)
    table(draft, "draft loops (all summarised rounds)", out)
    table(verify, "target pass + accept + commit (all summarised rounds)", out)


if __name__ == "__main__":
    main()
