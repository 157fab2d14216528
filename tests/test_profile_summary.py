"""CPU test of the profile summariser on a small synthetic set of rocprofv3 CSV files: kernel names are
recognised in mangled form, launches of the folded call and of per-layer calls stay apart by grid size, the
traffic counters are scaled by the copy calibration, and the roofline fraction in the summary is the one the
numbers give."""
import csv
import json
import os

from paper_2510_17777_amd import profile_summary as ps

SCORE = "_ZN2sv12_GLOBAL__N_112score_kernelIDF16_Li128ELb1ELb1EEEvNS_9ScoreArgsE"
ATTN = "_ZN2sv12_GLOBAL__N_125attn_partial_flash_kernelILi7EEEvNS_8AttnArgsEi"
COPY = "_ZN2sv12_GLOBAL__N_111copy_kernelEPK15HIP_vector_typeIjLj4EEPS2_m"
OTHER = "_ZN2at6native29vectorized_elementwise_kernelILi4EEEvv"


def _trace(path, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    cols = ["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp", "Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"]
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(cols)
        t = 1000
        for name, grid, dur_ns in rows:
            w.writerow(["KERNEL_DISPATCH", name, t, t + dur_ns, grid, 1, 1])
            t += dur_ns + 500


def _counters(path, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f, quoting=csv.QUOTE_NONNUMERIC)
        w.writerow(["Grid_Size", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for grid, name, counter, value in rows:
            w.writerow([grid, name, counter, value])


def test_kernel_names_are_recognised():
    assert ps.short_name(SCORE) == "score_kernel<stream,candidates>"
    assert ps.short_name(SCORE.replace("Lb1ELb1E", "Lb1ELb0E")) == "score_kernel<stream>"
    assert ps.short_name(ATTN) == "attn_partial_flash_kernel"
    assert ps.short_name("void sv::(anonymous namespace)::score_kernel<_Float16, 128, true, true>(sv::ScoreArgs)") \
        == "score_kernel<stream,candidates>"
    assert ps.short_name("sv::scores_filter_kernel(sv::ScoreArgs, int)") == "scores_filter_kernel"
    assert ps.short_name(OTHER) is None


def test_summaries_from_synthetic_csv(tmp_path):
    d = str(tmp_path)
    big, small = 5648384, 201728
    _trace(os.path.join(d, "trace", "t_kernel_trace.csv"),
           [(SCORE, big, 200_000), (SCORE, big, 210_000), (SCORE, small, 17_000), (ATTN, 172032, 40_000), (OTHER, 64, 5_000)])
    kb = 1438646272
    _counters(os.path.join(d, "fetch", "f_counter_collection.csv"),
              [(big, SCORE, "FETCH_SIZE", kb / 1024 / 2 * 1.01), (small, SCORE, "FETCH_SIZE", 25_000.0),
               (172032, ATTN, "FETCH_SIZE", 100_000.0)])
    _counters(os.path.join(d, "write", "w_counter_collection.csv"),
              [(big, SCORE, "WRITE_SIZE", 6_000.0), (small, SCORE, "WRITE_SIZE", 300.0), (172032, ATTN, "WRITE_SIZE", 2_500.0)])
    _counters(os.path.join(d, "lds", "l_counter_collection.csv"),
              [(big, SCORE, "SQ_LDS_IDX_ACTIVE", 1000.0), (big, SCORE, "SQ_LDS_BANK_CONFLICT", 100.0), (big, SCORE, "SQ_INSTS_LDS", 10.0)])
    _counters(os.path.join(d, "cal_f", "f_counter_collection.csv"), [(1 << 22, COPY, "FETCH_SIZE", 524288.0)])   # half the KiB
    _counters(os.path.join(d, "cal_w", "w_counter_collection.csv"), [(1 << 22, COPY, "WRITE_SIZE", 1048576.0)])
    bench = {"value": 270.0, "step_achieved_GBps": 6078.0, "step_hbm_frac": 0.76, "source_id": "abc123",
             "roofline": {"mean_us": 208.0, "bytes_per_launch": kb, "achieved": 6916.0, "frac": 0.8645}}
    open(os.path.join(d, "bench.json"), "w").write("warm-up noise\n" + json.dumps(bench) + "\n")

    st = ps.kernel_stats(os.path.join(d, "trace"))
    assert st[("score_kernel<stream,candidates>", big)][:2] == (2, 205.0)
    assert st[("score_kernel<stream,candidates>", small)][:2] == (1, 17.0)
    assert ps.largest_grid(st, "score_kernel") == ("score_kernel<stream,candidates>", big)
    assert all(k[0] != "vectorized_elementwise_kernel" for k in st)

    import sys
    argv, sys.argv = sys.argv, ["profile_summary", "--config", "4", "--dir", d, "--out", os.path.join(d, "out"), "--head", "deadbee"]
    try:
        ps.main()
    finally:
        sys.argv = argv
    trace_txt = open(os.path.join(d, "out", "decode_step_cfg4_kernel_trace.txt")).read()
    assert "source_id = abc123" in trace_txt and "git deadbee" in trace_txt
    # 1438646272 B in 205.0 us = 7017.8 GB/s = 87.7 % of 8 TB/s
    assert "avg 205.0 us -> 7017.8 GB/s = 87.7 % of 8 TB/s" in trace_txt
    traffic_txt = open(os.path.join(d, "out", "decode_step_cfg4_traffic_and_lds.txt")).read()
    assert "factor 2.000" in traffic_txt and "factor 1.000" in traffic_txt
    fetched = kb * 1.01
    assert "traffic_bytes_per_launch = %d" % round(fetched + 6000 * 1024) in traffic_txt
    assert "(x1.0100)" in traffic_txt
    # what bench.py reads back from the summary
    import bench
    root = bench.ROOT
    try:
        bench.ROOT = str(tmp_path)
        os.makedirs(os.path.join(str(tmp_path), "profiles"))
        os.replace(os.path.join(d, "out", "decode_step_cfg4_traffic_and_lds.txt"),
                   os.path.join(str(tmp_path), "profiles", "decode_step_cfg4_traffic_and_lds.txt"))
        val, src = bench.measured_traffic(4)
        assert val == round(fetched + 6000 * 1024) and "abc123" in src and "not measured in this run" in src
        assert bench.measured_traffic(2) == (None, None)
    finally:
        bench.ROOT = root
