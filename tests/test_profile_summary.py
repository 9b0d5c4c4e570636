"""The rocprofv3 trace condenser: rounds are cut at begin_round_k, a target pass at the kernel
that plans the verify rows, and the per-kernel averages are taken over the kept rounds only."""
import csv
import io
from contextlib import redirect_stdout

from paper_2405_19715_amd import profile_summary as PS


def _trace(path, n_rounds):
    t = 1000
    rows = []

    def add(name, dur):
        nonlocal t
        rows.append({"Kernel_Name": name, "Start_Timestamp": t, "End_Timestamp": t + dur})
        t += dur + 100
    add("void sd::(anonymous namespace)::gemm_bf16_tile<2, 2, 2, 2, 64, 2>(int)", 900)      # prompt pass
    for r in range(n_rounds):
        add("sd::(anonymous namespace)::begin_round_k(int)", 10)
        for _ in range(2):                                                                   # two draft steps
            add("sd::(anonymous namespace)::plan_draft_k(int)", 10)
            add("void sd::(anonymous namespace)::gemm_bf16_stream<1>(int)", 200)
        add("sd::(anonymous namespace)::plan_verify_k(int)", 10)
        for _ in range(3):
            add("void sd::(anonymous namespace)::gemm_bf16_stream<1>(int)", 700 if r >= 1 else 5000)
        add("void sd::(anonymous namespace)::gemm_bf16_stripe<5>(int)", 300)
        add("sd::(anonymous namespace)::commit_k(int)", 10)
    with open(path, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=list(rows[0]))
        w.writeheader()
        w.writerows(rows)


def test_summary_counts_rounds_and_averages(tmp_path):
    p = tmp_path / "trace.csv"
    _trace(p, 4)
    out = io.StringIO()
    with redirect_stdout(out):
        PS.main([str(p), "--skip-rounds", "1"])
    text = out.getvalue()
    assert "rounds summarised: 3 (first 1 skipped)" in text
    assert "draft steps: 6" in text
    # the slow first round is skipped: the target pass's GEMM averages 0.70 us over 9 launches
    line = [l for l in text.splitlines() if "gemm_bf16_stream<1>" in l][-1]
    assert "calls      9" in line and "avg      0.70 us" in line
    # the weight-streaming kernels of the target pass also get one line together: (9 * 700 + 3 * 300) / 12 ns
    line = [l for l in text.splitlines() if "all weight-streaming GEMMs" in l][-1]
    assert "calls     12" in line and "avg      0.60 us" in line
    assert "prompt pass" in text and "gemm_bf16_tile<2, 2, 2, 2, 64, 2>" in text


def test_by_grid_averages_per_kernel_and_grid(tmp_path):
    p = tmp_path / "trace.csv"
    rows = []
    for i, (name, gx, gy, dur) in enumerate([("sd::(anonymous namespace)::accept_k(float)", 1024, 1, 100),
                                             ("sd::(anonymous namespace)::accept_k(float)", 1024, 1, 300),
                                             ("sd::(anonymous namespace)::accept_k(float)", 65536, 1, 500),
                                             ("void sd::(anonymous namespace)::row_stats_k<true, false>(int)", 33792, 64, 4000),
                                             ("void other_k(int)", 64, 1, 7)]):
        rows.append({"Kernel_Name": name, "Start_Timestamp": 1000 * i, "End_Timestamp": 1000 * i + dur,
                     "Grid_Size_X": gx, "Grid_Size_Y": gy, "Workgroup_Size_X": 1024, "Workgroup_Size_Y": 1})
    with open(p, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=list(rows[0]))
        w.writeheader()
        w.writerows(rows)
    out = io.StringIO()
    with redirect_stdout(out):
        PS.main([str(p), "--by-grid", "accept_k,row_stats_k"])
    lines = out.getvalue().splitlines()
    assert len(lines) == 3 and "other_k" not in out.getvalue()
    assert "grid (  1,   1)  calls    2  avg     0.20 us" in lines[0]
    assert "grid ( 64,   1)  calls    1  avg     0.50 us" in lines[1]
    assert "row_stats_k<true, false>" in lines[2] and "grid ( 33,  64)" in lines[2] and "4.00 us" in lines[2]
