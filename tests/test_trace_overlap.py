"""The stream-overlap analysis of a rocprofv3 kernel trace, on a synthetic trace."""
import csv

import trace_overlap


def _write(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kind", "Kernel_Name", "Start_Timestamp", "End_Timestamp"])
        for name, s, e in rows:
            w.writerow(["KERNEL_DISPATCH", name, s, e])


def test_overlap_fraction_on_a_hand_made_trace(tmp_path):
    gemm = "Cijk_Ailk_Bljk_something"
    sync = "void xs::reduce_sgd_kernel<8, 0, false, true, true>(...)"
    rows = [
        (gemm, 0, 1_000_000), (gemm, 1_000_000, 2_000_000),          # compute: [0, 2 ms)
        (sync, 500_000, 900_000),                                     # wholly inside: 0.4 ms
        (sync, 1_800_000, 2_200_000),                                 # half inside: 0.2 of 0.4 ms
        ("void at::native::something()", 100, 200),                   # neither kind: ignored
        (sync, 50_000_000, 50_400_000),                               # far from any compute: a
        ("alu_kernel(float*, unsigned int, float, float)", 90_000_000, 91_000_000),
        (sync, 90_200_000, 90_300_000),                               # inside the stand-in: 0.1 ms
    ]
    p = tmp_path / "t_kernel_trace.csv"
    _write(p, rows)
    r = trace_overlap.analyse(str(p))
    assert r["sync_kernels_total"] == 4 and r["sync_kernels_in_crossover_phase"] == 3
    assert abs(r["sync_time_ms"] - 0.9) < 1e-9
    assert abs(r["sync_time_inside_compute_ms"] - 0.7) < 1e-9
    assert abs(r["stream_overlap_fraction"] - 0.7 / 0.9) < 1e-12


def test_gemm_time_lost_beside_sync(tmp_path):
    gemm = "Cijk_Ailk_Bljk_something"
    sync = "void xs::copy_kernel<false>(...)"
    rows = [(gemm, 0, 800_000), (gemm, 800_000, 1_600_000), (gemm, 1_600_000, 2_400_000),   # alone: 0.8 ms
            (gemm, 2_400_000, 3_400_000), (gemm, 3_400_000, 4_500_000),                      # beside: 1.0, 1.1 ms
            (sync, 2_500_000, 4_400_000),
            (gemm, 4_500_000, 5_300_000)]
    p = tmp_path / "t_kernel_trace.csv"
    _write(p, rows)
    r = trace_overlap.analyse(str(p))
    assert r["gemm_kernels_alone"] == 4 and r["gemm_kernels_beside_sync"] == 2
    assert abs(r["gemm_median_alone_us"] - 800.0) < 1e-9
    assert abs(r["gemm_time_lost_beside_sync_ms"] - 0.5) < 1e-9
    assert abs(r["sync_busy_time_ms"] - 1.9) < 1e-9


def test_gemm_time_lost_is_summed_over_kernel_names(tmp_path):
    a, b, c = "Cijk_small_tile", "Cijk_large_tile", "Cijk_never_beside"
    sync = "void xs::gather_reduce_sgd_kernel<4>(...)"
    rows = [(a, 0, 100_000), (a, 100_000, 200_000), (b, 200_000, 500_000), (c, 500_000, 900_000),   # alone
            (a, 1_000_000, 1_150_000),                      # beside: +0.05 ms over its own 0.1 ms
            (b, 1_150_000, 1_850_000),                      # beside: +0.4 ms over its own 0.3 ms
            (sync, 1_010_000, 1_800_000)]
    p = tmp_path / "t_kernel_trace.csv"
    _write(p, rows)
    r = trace_overlap.analyse(str(p))
    assert abs(r["gemm_time_lost_beside_sync_ms"] - 0.45) < 1e-9
    assert r["gemm_kernel_with_most_time_beside_sync"] == b
    assert r["gemm_kernels_alone"] == 1 and r["gemm_kernels_beside_sync"] == 1
    assert abs(r["gemm_median_alone_us"] - 300.0) < 1e-9 and abs(r["gemm_median_beside_sync_us"] - 700.0) < 1e-9


def test_merge_and_classify():
    assert trace_overlap.merge([(5, 7), (0, 3), (2, 4), (7, 9)]) == [(0, 4), (5, 9)]
    assert trace_overlap.classify("void xs::copy_kernel<false>(...)") == "sync"
    assert trace_overlap.classify("Cijk_x") == "compute"
    assert trace_overlap.classify("hipMemset") is None
