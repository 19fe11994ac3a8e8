"""Host logic of bench.py that needs no GPU: the text summary of rocprofv3 CSV output and the stored traffic."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_kernel_trace_summary_groups_by_kernel_and_grid_and_splits_populations(tmp_path):
    d = tmp_path / "run" / "node"
    d.mkdir(parents=True)
    rows = ["Kernel_Name,Grid_Size,Start_Timestamp,End_Timestamp"]
    for i in range(4):                                                  # the same grid, two populations of durations
        rows.append(f"void (anonymous namespace)::scan<4>(Args),131072,{1000 * i},{1000 * i + 100000}")   # 100 us
    for i in range(2):
        rows.append(f"void (anonymous namespace)::scan<4>(Args),131072,{9000 + i},{9000 + i + 10000}")    # 10 us
    rows.append("void (anonymous namespace)::scan<4>(Args),131072,0,30000")                               # 30 us: a third population
    rows.append("void other(int),256,0,5000")                                                              # 5 us
    (d / "1_kernel_trace.csv").write_text("\n".join(rows) + "\n")
    text = bench.summarize_rocprof(str(tmp_path / "run"), "cmd --flag")
    lines = text.splitlines()
    assert lines[0] == "command: cmd --flag"
    long_ = next(l for l in lines if "scan<4> [population 1 of 3]" in l).replace("[population 1 of 3]", "").split()
    mid = next(l for l in lines if "scan<4> [population 2 of 3]" in l).replace("[population 2 of 3]", "").split()
    short = next(l for l in lines if "scan<4> [population 3 of 3]" in l).replace("[population 3 of 3]", "").split()
    assert mid[-7:-1] == ["131072", "1", "30.0", "30.00", "30.00", "30.00"]
    other = next(l for l in lines if l.strip().startswith("other")).split()
    # name [tag] grid calls total average min max share
    assert long_[-7:-1] == ["131072", "4", "400.0", "100.00", "100.00", "100.00"]
    assert short[-7:-1] == ["131072", "2", "20.0", "10.00", "10.00", "10.00"]
    assert other[-7:-1] == ["256", "1", "5.0", "5.00", "5.00", "5.00"]
    assert abs(float(long_[-1].rstrip("%")) - 100 * 400 / 455) < 0.01


def test_counter_summary_gives_mean_min_max_per_dispatch(tmp_path):
    d = tmp_path / "pmc"
    d.mkdir()
    rows = ["Kernel_Name,Grid_Size_X,Grid_Size_Y,Grid_Size_Z,Counter_Name,Counter_Value"]
    for v in (10.0, 20.0, 60.0):
        rows.append(f"void k(float*),64,2,1,FETCH_SIZE,{v}")
    (d / "7_counter_collection.csv").write_text("\n".join(rows) + "\n")
    text = bench.summarize_rocprof(str(d), "")
    line = next(l for l in text.splitlines() if "FETCH_SIZE" in l).split()
    assert line == ["k", "128", "FETCH_SIZE", "3", "30.0", "10.0", "60.0"]
    assert text.splitlines()[0] == "command: (not given)"


def test_stored_traffic_reads_the_committed_summary():
    t, src = bench.stored_traffic("cfg1")
    assert t is not None and 1e8 < t < 1e9            # bytes per scan launch at cfg1: a few hundred MB
    assert src.startswith("stored: profiles/adc_scan_traffic_cfg1.txt") and "not measured in this run" in src
    t, src = bench.stored_traffic("no_such_workload")
    assert t is None and "no stored counter summary" in src
