"""Stream-overlap fraction from a rocprofv3 kernel trace (CSV).

    python trace_overlap.py <prefix>_kernel_trace.csv

For the crossover schedule (arXiv 2103.07974, Section 2.1) the question is how much of the
time the synchronisation kernels run falls inside the time the other task's compute kernels
run:  sum |sync interval ∩ union(compute intervals)| / sum |sync interval|.
Kernels of libxs.so (namespace xs::) count as synchronisation; GEMM kernels (names starting
with Cijk_) and the arithmetic-only stand-in of bench_standin.hip count as compute.
Only the part of the trace where both kinds appear within one millisecond of each other is
used, so that stand-alone timing loops in the same trace do not dilute the figure.
It also reports what the overlap costs the computation: the GEMM kernels that ran while a
sync kernel was running against the median of those of the same name that ran alone (time
lost, summed over the kernel names), beside the time the sync stream was busy.
"""
from __future__ import annotations

import csv
import sys
from typing import List, Tuple


def classify(name: str) -> str | None:
    if "alu_kernel" in name or name.startswith("Cijk_"):
        return "compute"
    if "xs::" in name:
        return "sync"
    return None


def merge(iv: List[Tuple[int, int]]) -> List[Tuple[int, int]]:
    out: List[Tuple[int, int]] = []
    for s, e in sorted(iv):
        if out and s <= out[-1][1]:
            out[-1] = (out[-1][0], max(out[-1][1], e))
        else:
            out.append((s, e))
    return out


def overlap_with(iv: Tuple[int, int], merged: List[Tuple[int, int]]) -> int:
    s, e = iv
    tot = 0
    for a, b in merged:
        if b <= s:
            continue
        if a >= e:
            break
        tot += min(e, b) - max(s, a)
    return tot


def analyse(path: str, slack_ns: int = 1_000_000):
    sync, comp, comp_named = [], [], []
    for r in csv.DictReader(open(path)):
        kind = classify(r["Kernel_Name"])
        if kind is None:
            continue
        iv = (int(r["Start_Timestamp"]), int(r["End_Timestamp"]))
        (sync if kind == "sync" else comp).append(iv)
        if kind == "compute":
            comp_named.append((iv, r["Kernel_Name"]))
    comp_m = merge(comp)
    # widen compute intervals by the slack to decide which sync kernels belong to the crossover phase
    near = merge([(a - slack_ns, b + slack_ns) for a, b in comp_m])
    used = [iv for iv in sync if overlap_with(iv, near) > 0]
    tot = sum(e - s for s, e in used)
    inside = sum(overlap_with(iv, comp_m) for iv in used)
    # what the overlap costs the computation: per GEMM kernel name, the launches that ran while
    # a sync kernel was running against the median duration of those of that name that ran
    # alone (a trace may also hold the timing runs of other hipBLASLt algorithms: names with no
    # launch beside a sync kernel are left out); the "main" kernel is the name with the most
    # time beside sync kernels
    sync_m = merge(used)
    by_name = {}
    for iv, nm in comp_named:
        if nm.startswith("Cijk_"):
            by_name.setdefault(nm, ([], []))[1 if overlap_with(iv, sync_m) > 0 else 0].append(iv[1] - iv[0])
    lost, main, main_time = None, None, -1
    for nm, (alone_d, beside_d) in by_name.items():
        if not beside_d:
            continue
        if alone_d:
            base_nm = sorted(alone_d)[len(alone_d) // 2]
            lost = (lost or 0) + sum(d - base_nm for d in beside_d)
        if sum(beside_d) > main_time:
            main, main_time = nm, sum(beside_d)
    alone, beside = (sorted(by_name[main][0]), by_name[main][1]) if main else ([], [])
    base = alone[len(alone) // 2] if alone else None
    return {"sync_kernels_in_crossover_phase": len(used), "sync_kernels_total": len(sync),
            "sync_time_ms": tot / 1e6, "sync_time_inside_compute_ms": inside / 1e6,
            "stream_overlap_fraction": inside / tot if tot else None,
            "gemm_kernels_alone": len(alone), "gemm_median_alone_us": base / 1e3 if base else None,
            "gemm_kernels_beside_sync": len(beside),
            "gemm_median_beside_sync_us": sorted(beside)[len(beside) // 2] / 1e3 if beside else None,
            "gemm_kernel_with_most_time_beside_sync": main[:60] if main else None,
            "gemm_time_lost_beside_sync_ms": lost / 1e6 if lost is not None else None,
            "sync_busy_time_ms": sum(e - s for s, e in sync_m) / 1e6}


if __name__ == "__main__":
    if len(sys.argv) != 2:
        sys.exit(__doc__)
    for k, v in analyse(sys.argv[1]).items():
        print(f"{k}: {v}")
