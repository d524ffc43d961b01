#!/usr/bin/env python3
"""Benchmark of the fused gradient-synchronisation path on one MI355X.

Default run (what the one JSON line reports):
  step      one whole synchronisation of the VGG-16-shaped gradient set on one stream, inputs
            resident in HBM: the W = 8 packs (one launch), the fused reduce + SGD, the unpack.
            `value` = (W*s + 16) * N bytes (W replica buckets, parameters and momentum read,
            parameters and momentum written) / time of the whole step.
  roofline  the fused reduce + SGD kernel of that step alone, HIP events around each launch
            inside the timed region; `roofline_by_config` repeats it stand-alone for the
            ResNet-50-, VGG-16- and BERT-large-shaped sets (>= 10 warm-up, >= 50 timed launches).
  crossover the two-stream schedule of Algorithm 1 (ResNet-50- and VGG-16-shaped tasks beside
            the configured chain of bf16 GEMMs): the end-to-end hidden fraction
            1 - (T_cross - T_comp) / (T_serial - T_comp) leads; everything else is labelled.
  cpu_baseline  the C oracle's single-precision reduce + SGD on a slice of the same buckets,
            one thread and all host cores.

Other modes (used for the summaries under profiles/):
  --kernels-only W      stand-alone launches of every kernel of workload W, nothing else
                        (rocprofv3 --kernel-trace --stats)
  --traffic-probe W     a calibration copy, then a few launches of every kernel of workload W
                        (rocprofv3 --pmc)
  --stream-ceiling      plain 1:1 copy and 10-read : 2-write streaming kernels (attainable HBM rate)
  --crossover-sweep     the crossover pair under CU partitions and launch settings, one child
                        process per case (hipBLASLt reads its stream-K grid size once per process)
  --crossover-only      one short two-stream run and nothing else (rocprofv3 --kernel-trace)
  --power               board power and a clock proxy beside the GEMM chain / the sync kernels
  --footprint           which register footprints are placed beside each GEMM algorithm's workgroups
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "fused grad-sync GB/s + % HBM roofline; crossover sync-hidden fraction (1 GPU)"
# figures that are NOT measured by this run: copied from the committed rocprofv3 summaries
FROM_PROFILES = {
    "note": "copied from committed rocprofv3 summaries, not measured in this run",
    "reduce_sgd_vgg16_hbm_bytes_per_launch": {
        "value": 6641046995, "algorithmic": 6641162112,
        "file": "profiles/hbm_traffic_pmc_all_kernels.md"},
}


def _median(xs_):
    s = sorted(xs_)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def _stats(ms):
    return {"avg_launch_ms": sum(ms) / len(ms), "median_launch_ms": _median(ms), "min_launch_ms": min(ms),
            "launches": len(ms)}


def _events(n):
    import torch
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


# --------------------------------------------------------------------------- headline step
def time_steps(tasks, steps, warmup, stream, fused_unpack=False):
    """K whole steps on `stream`, rotating over the buffer sets; events around the reduce + SGD
    kernel of each step.  Returns (ms per step, [kernel ms])."""
    import torch
    from paper_2103_07974_amd import xs
    ev = _events(steps)

    def one(task, pair=None):
        w = task.workload
        xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets, None, stream)
        if pair:
            pair[0].record(stream)
        if fused_unpack:
            xs.fused_reduce_sgd_unpack(task.gplan, task.buckets, task.params, task.momentum, task.param_table,
                                       w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale, stream=stream)
        else:
            xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum,
                                w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale, stream=stream)
        if pair:
            pair[1].record(stream)
        if not fused_unpack:
            xs.fuse_unpack(task.pplan, task.params, task.param_table, stream)

    with torch.cuda.stream(stream):
        for i in range(warmup):
            one(tasks[i % len(tasks)])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            one(tasks[i % len(tasks)], ev[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, [a.elapsed_time(b) for a, b in ev]


def timed_launches(fn, stream, launches=50, warmup=10):
    """HIP events on the launch stream around each of `launches` calls of fn(i), after warm-up."""
    import torch
    ts = []
    with torch.cuda.stream(stream):
        for i in range(warmup):
            fn(i)
        stream.synchronize()
        for i in range(launches):
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(stream); fn(i); b.record(stream); b.synchronize()
            ts.append(a.elapsed_time(b))
    return ts


def reduce_roofline(tasks, stream, launches=50, warmup=10):
    """The fused reduce + SGD kernel alone (rotating over the buffer sets)."""
    from paper_2103_07974_amd import xs
    w = tasks[0].workload

    def fn(i):
        t = tasks[i % len(tasks)]
        xs.fused_reduce_sgd(t.buckets, t.n_bucket, t.params, t.momentum, w.lr, w.momentum,
                            w.weight_decay, 1.0 / w.loss_scale, stream=stream)
    ms = timed_launches(fn, stream, launches, warmup)
    nbytes = tasks[0].reduce_bytes()
    st = _stats(ms)
    gt = {"f32": 0, "f16": 1, "bf16": 2}[w.grad_dtype]
    return {"bound": "hbm", "kernel": f"xs::reduce_sgd_kernel<{w.W}, {gt}, false, true, true, false, false>",
            "achieved": nbytes / st["avg_launch_ms"] / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": nbytes / st["avg_launch_ms"] / 1e6 / HBM_PEAK_GBS, "bytes_per_launch": nbytes,
            "bytes_per_element": w.W * w.grad_bytes + 16, "elements": w.n_elems, **st}


def other_kernels(tasks, stream, launches=30, warmup=6):
    """Medians of the path's other kernels on one workload (not part of the 75 % bar)."""
    from paper_2103_07974_amd import xs
    t0 = tasks[0]; w = t0.workload
    out = {}

    def med(fn):
        return _median(timed_launches(fn, stream, launches, warmup))

    def T(i):
        return tasks[i % len(tasks)]
    ms = med(lambda i: xs.fuse_pack(T(i).gplan, T(i).grad_tables[i % w.W], T(i).buckets[i % w.W], None, stream))
    out["pack_one_replica"] = {"ms": ms, "GBs": t0.pack_bytes() / ms / 1e6}
    ms = med(lambda i: xs.fuse_pack_many(T(i).gplan, T(i).grad_tables, T(i).buckets, None, stream))
    out["pack_all_replicas_one_launch"] = {"ms": ms, "GBs": w.W * t0.pack_bytes() / ms / 1e6,
                                           "frac_of_hbm_peak": w.W * t0.pack_bytes() / ms / 1e6 / HBM_PEAK_GBS}
    ms = med(lambda i: xs.fuse_unpack(T(i).pplan, T(i).params, T(i).param_table, stream))
    out["unpack"] = {"ms": ms, "GBs": t0.unpack_bytes() / ms / 1e6,
                     "frac_of_hbm_peak": t0.unpack_bytes() / ms / 1e6 / HBM_PEAK_GBS}
    ms = med(lambda i: xs.fused_reduce_sgd_unpack(T(i).gplan, T(i).buckets, T(i).params, T(i).momentum,
                                                  T(i).param_table, w.lr, w.momentum, w.weight_decay,
                                                  1.0 / w.loss_scale, stream=stream))
    nb = t0.reduce_bytes() + 4 * w.n_elems
    out["reduce_sgd_with_fused_unpack"] = {"ms": ms, "GBs": nb / ms / 1e6, "frac_of_hbm_peak": nb / ms / 1e6 / HBM_PEAK_GBS,
                                           "bytes_per_element": w.W * w.grad_bytes + 20}
    ms = med(lambda i: xs.fused_gather_reduce_sgd(T(i).gplan, T(i).gather_table, w.W, T(i).params, T(i).momentum,
                                                  w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale,
                                                  param_tensor_ptrs=T(i).param_table, stream=stream))
    nb = t0.gather_bytes(True)
    out["gather_form_whole_step"] = {"ms": ms, "GBs": nb / ms / 1e6, "frac_of_hbm_peak": nb / ms / 1e6 / HBM_PEAK_GBS,
                                     "GBs_by_headline_formula": t0.reduce_bytes() / ms / 1e6}
    table = xs.tensor_hparams_table([(w.lr, w.momentum, w.weight_decay) if len(s) > 1
                                     else (2 * w.lr, w.momentum, 0.0) for s in w.shapes])
    ms = med(lambda i: xs.fused_reduce_sgd_pt(T(i).gplan, T(i).buckets, T(i).params, T(i).momentum, table,
                                              1.0 / w.loss_scale, stream=stream))
    out["reduce_sgd_param_groups"] = {"ms": ms, "GBs": t0.reduce_bytes() / ms / 1e6,
                                      "frac_of_hbm_peak": t0.reduce_bytes() / ms / 1e6 / HBM_PEAK_GBS}
    return out


def time_overflow_skip(task, stream, reps=8):
    """Loss-scale overflow (the mixed-precision workload with non-finite gradients in one
    replica): the W packs with detection raise the flag, the reduce + SGD launched behind them
    returns at once and leaves the state untouched."""
    import torch
    from paper_2103_07974_amd import xs
    w = task.workload
    g = torch.Generator(device="cuda"); g.manual_seed(w.seed + 999)
    for t in task.grads[0]:           # about 0.1 % of replica 0's elements become +inf
        k = max(1, t.numel() // 1000)
        idx = torch.randint(0, t.numel(), (k,), generator=g, device="cuda")
        t.view(-1)[idx] = float("inf")
    x_before = task.params[:4096].clone()
    pack_ms, red_ms = [], []
    with torch.cuda.stream(stream):
        for i in range(reps + 2):
            task.found_inf.zero_()
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
            xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets, task.found_inf, stream)
            e[1].record(stream)
            xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum, w.lr,
                                w.momentum, w.weight_decay, 1.0 / w.loss_scale,
                                found_inf=task.found_inf, stream=stream)
            e[2].record(stream); e[2].synchronize()
            if i >= 2:
                pack_ms.append(e[0].elapsed_time(e[1])); red_ms.append(e[1].elapsed_time(e[2]))
    assert int(task.found_inf.item()) == 1 and torch.equal(task.params[:4096], x_before)
    return {"pack_all_replicas_with_detection_ms": _median(pack_ms),
            "pack_all_replicas_with_detection_GBs": w.W * task.pack_bytes() / _median(pack_ms) / 1e6,
            "skipped_reduce_sgd_ms": _median(red_ms), "flag_raised": True}


# --------------------------------------------------------------------------- compute stand-ins
class GemmChain:
    """The configured compute stand-in: `chain` bf16 GEMMs Y <- Y @ B of dim^3 on one stream,
    through hipBLASLt with an explicit algorithm (index 0 is the library's own first choice,
    the kernel torch.matmul runs)."""

    def __init__(self, dim=8192, chain=16, max_algos=16, seed=20210407):
        import torch
        import bench_standin as bs
        g = torch.Generator(device="cuda"); g.manual_seed(seed)
        self.B = (torch.randn(dim, dim, generator=g, device="cuda") / dim ** 0.5).to(torch.bfloat16)
        self.Y = [torch.randn(dim, dim, generator=g, device="cuda").to(torch.bfloat16) for _ in range(2)]
        self.Y_init = self.Y[0].clone()
        self.gemm = bs.Gemm(dim, max_algos)
        self.dim, self.chain = dim, chain
        self.label = f"{chain}x[{dim}x{dim}]@[{dim}x{dim}] bf16"

    def enqueue(self, algo, stream_ptr, source=None, n=None):
        """GEMM k reads the result of GEMM k-1; the first reads the seeded matrix, which is never
        written.  (Left to run on from its own output, Y @ B @ B ... overflows to inf/NaN after a
        few hundred products, and a GEMM on such operands draws less power and runs 20 % faster
        on this chip.)"""
        src = self.Y_init if source is None else source
        for k in range(self.chain if n is None else n):
            dst = self.Y[k & 1]
            self.gemm.run(algo, src, self.B, dst, stream_ptr)
            src = dst

    def fn(self, algo=0):
        def compute(stream_ptr):
            self.enqueue(algo, stream_ptr)
        return compute

    def time_algo(self, algo, stream, reps=2):
        import torch
        f = self.fn(algo)
        with torch.cuda.stream(stream):
            f(stream.cuda_stream)
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                f(stream.cuda_stream)
            b.record(stream); b.synchronize()
        return a.elapsed_time(b) / reps

    def admits_neighbours(self, algo, cs, ss, vgprs=48):
        """Can a 4-wave workgroup of `vgprs` registers per lane and an 82 KiB LDS reservation be
        placed on a compute unit while this algorithm's workgroups are resident?  (A launch of
        such workgroups beside a running chain finishes within a fraction of one GEMM if so,
        and only at the next kernel boundary if not.)"""
        import torch
        import bench_standin as bs
        out = torch.zeros(1024, dtype=torch.int32, device="cuda"); ts = torch.zeros(1024, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        f1 = torch.cuda.Event(enable_timing=True)
        e0.record(cs)
        self.enqueue(algo, cs, n=4)
        e1.record(cs)
        ss.wait_event(e0)
        bs.footprint(out, ts, 1024, 256, 82 * 1024, vgprs, 100, ss)
        f1.record(ss)
        torch.cuda.synchronize()
        one_gemm = e0.elapsed_time(e1) / 4
        return e0.elapsed_time(f1) < 0.5 * one_gemm

    def choose_for_sharing(self, cs, ss, tolerance=1.10):
        """Among the algorithms within `tolerance` of the fastest, the first that leaves room
        for a small neighbour on every compute unit; else the fastest."""
        times = {a: self.time_algo(a, cs) for a in range(self.gemm.n_algos)}
        best = min(times.values())
        for a in sorted(times, key=times.get):
            if times[a] <= tolerance * best and self.admits_neighbours(a, cs, ss):
                return a, times
        return min(times, key=times.get), times


def alu_standin(target_ms):
    """One arithmetic-only kernel of ordinary occupancy and no memory traffic (256 workgroups of
    256 lanes) calibrated to last target_ms: the kind of kernel that is not at the board's
    power limit and leaves wave slots free."""
    import torch
    import bench_standin as bs
    sink = torch.zeros(256, device="cuda")
    probe_iters = 100000
    a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
    bs.alu(256, probe_iters, sink); torch.cuda.synchronize()
    a0.record(); bs.alu(256, probe_iters, sink); a1.record(); a1.synchronize()
    iters = max(1000, int(probe_iters * target_ms / a0.elapsed_time(a1)))

    def compute(stream_ptr):
        bs.alu(256, iters, sink, stream_ptr)
    return compute, f"one arithmetic-only kernel, 256x256 lanes, {iters} x 8 multiply-adds per lane"


# --------------------------------------------------------------------------- crossover
def crossover_run(tasks, computes, label, T=20, rounds=5, form="packs", tuning=None, streams=None,
                  cross_only=False, t_comp_reference=None):
    """N tasks alternate as in Algorithm 1: one computes while the task that has just sent its
    gradients is synchronised on the second stream.  Three schedules of the same work:
      T_comp    the N*T computations only, compute stream
      T_serial  computation and synchronisation strictly alternating on one stream (the
                synchronisation with its default, fastest launch settings)
      T_cross   xs_crossover_iteration on two streams (synchronisations launched with `tuning`)
    hidden = 1 - (T_cross - T_comp) / (T_serial - T_comp) charges every slow-down of the
    computation to the synchronisation.  The chip's clocks drift with its thermal and power
    state by more than the difference being measured, so the three schedules are run
    round-robin and every figure is a median over the rounds."""
    import torch
    from paper_2103_07974_amd import xs
    kw = {"fused_gather": form == "gather", "fused_unpack": form == "fused_unpack"}
    cs, ss = streams if streams is not None else (torch.cuda.Stream(), torch.cuda.Stream())
    spans = None        # while a list: (task, start event, end event) of every computation on the compute stream

    def timed(i, c):
        def compute(stream_ptr):
            if spans is None or stream_ptr != cs.cuda_stream:
                return c(stream_ptr)
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record(cs); c(stream_ptr); e1.record(cs)
            spans.append((i, e0, e1))
        return compute
    apps = [t.make_app(timed(i, c), tuning=tuning, **kw) for i, (t, c) in enumerate(zip(tasks, computes))]
    alone = apps if tuning is None else [t.make_app(c, **kw) for t, c in zip(tasks, computes)]
    N = len(apps)

    def run_cross(record=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(T):
            xs.crossover_iteration(apps, cs, ss)
            if record is not None and t > 0:
                es = torch.cuda.Event(enable_timing=True); ec = torch.cuda.Event(enable_timing=True)
                es.record(ss); ec.record(cs)
                record.append((es, ec))
        xs.crossover_finish(apps, ss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_serial():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(T):
            for i in range(N):
                computes[i](cs.cuda_stream)
                alone[i].sync(cs)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_comp():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(T):
            for i in range(N):
                computes[i](cs.cuda_stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_sync(app, n=10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            app.sync(ss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def run_one_compute(i, n=3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            computes[i](cs.cuda_stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    names = {"packs": "W packs (1 launch), reduce+SGD, unpack", "fused_unpack": "W packs (1 launch), reduce+SGD+unpack (1 kernel)",
             "gather": "gather+reduce+SGD+views (1 kernel)"}
    if cross_only:       # for kernel tracing: nothing but the two-stream schedule itself
        run_cross()
        ms = run_cross()
        for a in set(apps + alone):
            a.destroy()
        return {"T": T, "n_tasks": N, "compute": label, "t_cross_ms": ms, "sync_kernels": names[form]}
    for _ in range(2):
        run_comp(); run_serial(); run_cross()
    rows, rec = [], []
    for r in range(rounds):
        rows.append((run_comp(), run_serial(), run_cross(rec if r == rounds - 1 else None)))
    t_comp, t_serial, t_cross = (_median([x[k] for x in rows]) for k in range(3))
    per_round = [1.0 - (x[2] - x[0]) / (x[1] - x[0]) for x in rows if x[1] > x[0]]
    sync_alone = [run_sync(a) for a in alone]
    comp_alone = [run_one_compute(i) for i in range(N)]
    sum_sync = t_serial - t_comp
    late = sum(1 for es, ec in rec if ec.elapsed_time(es) > 0)
    # Section 1, first contribution: no synchronisation delay as long as every task's
    # synchronisation fits under the other tasks' computations; the schedule then lasts
    # T * sum(C_i) + M_last (closed form of the timeline model)
    fits = all(sync_alone[i] <= sum(comp_alone) - comp_alone[i] for i in range(N)) if N > 1 else False
    res = {
        "T": T, "n_tasks": N, "compute": label, "sync_kernels": names[form], "rounds": rounds,
        "end_to_end_hidden_fraction": 1.0 - (t_cross - t_comp) / sum_sync if sum_sync > 0 else None,
        "hidden_fraction_median_of_rounds": _median(per_round) if per_round else None,
        "hidden_fraction_per_round": per_round,
        "speedup_vs_serial": t_serial / t_cross,
        "t_comp_ms": t_comp, "t_serial_ms": t_serial, "t_cross_ms": t_cross, "sum_sync_ms": sum_sync,
        "sync_alone_ms": sync_alone, "compute_alone_ms": comp_alone,
        "comm_comp_ratio": [sync_alone[i] / comp_alone[(i + 1) % N] for i in range(N)],
        "no_task_waits_model_T_cross_ms": (T * sum(comp_alone) + sync_alone[-1]) if fits else None,
        "iterations_whose_sync_outlasted_the_compute_beside_it": late, "of_iterations": len(rec),
    }
    if t_comp_reference is not None and sum_sync > 0:
        # the same schedule charged against the computation on an unrestricted stream
        res["t_comp_unrestricted_ms"] = t_comp_reference
        res["hidden_fraction_vs_unrestricted_compute"] = \
            1.0 - (t_cross - t_comp_reference) / (t_serial - t_comp)
    if N == 2:
        # Per task (two tasks): what task i's synchronisations cost the schedule = how much
        # longer the other task's computations were while they ran beside them, plus how long
        # task i's own next computation had to wait (the gap in front of it on the compute
        # stream); hidden_i = 1 - cost_i / (number of overlapped synchronisations * M_i alone).
        spans = []
        run_cross()
        sp, spans = spans, None
        cost = [0.0, 0.0]
        n_sync = [0, 0]
        for k in range(1, len(sp)):                 # every computation but the first runs beside the
            i, e0, e1 = sp[k]                       # synchronisation of the task that computed before it
            other = 1 - i
            n_sync[other] += 1
            cost[other] += max(0.0, e0.elapsed_time(e1) - comp_alone[i])       # beside task `other`'s sync
            cost[i] += max(0.0, sp[k - 1][2].elapsed_time(e0))                   # waiting for its own sync
        res["per_task"] = [{"sync_alone_ms": sync_alone[i], "synchronisations_counted": n_sync[i],
                            "cost_to_the_schedule_ms": cost[i],
                            "hidden_fraction": 1.0 - cost[i] / (n_sync[i] * sync_alone[i]) if n_sync[i] else None}
                           for i in range(2)]
    for a in set(apps + alone):
        a.destroy()
    return res


def crossover_case(spec):
    """One case of the sweep in a process of its own (argv: JSON).  Keys: form, k (compute
    units per XCD reserved for the sync stream; 0 = no partition), one_sided, algo, tuning
    ("default" | "beside"), T."""
    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); bs.lib(); torch.cuda.set_device(0); torch.zeros(1, device="cuda")
    gc = GemmChain()
    ta = harness.make_task(wl.RESNET50, "cuda"); tb = harness.make_task(wl.VGG16, "cuda")
    full_c, full_s = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        gc.time_algo(0, full_c)
    algo = spec.get("algo", 0)
    if algo == "share":
        algo, _ = gc.choose_for_sharing(full_c, full_s)
    f = gc.fn(algo)
    k = spec.get("k", 0)
    T = spec.get("T", 10)
    streams, ref, census = (full_c, full_s), None, None
    if k:
        sw, cw = bs.sync_and_compute_masks(k)
        s_masked = bs.MaskedStream(sw)
        c_stream = full_c if spec.get("one_sided") else bs.MaskedStream(cw).stream
        streams = (c_stream, s_masked.stream)
        census = {"sync_stream_compute_units": len(bs.census(4096, 2000, s_masked.stream)),
                  "compute_stream_compute_units": len(bs.census(8192, 2000, c_stream))}
        ref = _median([gc.time_algo(algo, full_c, reps=4) for _ in range(3)]) * 2 * T
    tuning = xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE) if spec.get("tuning") == "beside" else None
    r = crossover_run([ta, tb], [f, f], gc.label, T=T, rounds=spec.get("rounds", 5),
                      form=spec.get("form", "packs"), tuning=tuning, streams=streams, t_comp_reference=ref)
    r["case"] = spec
    r["gemm_algorithm_index"] = algo
    r["gemm_workgroups_per_launch"] = int(os.environ.get("TENSILE_STREAMK_FIXED_GRID", "256"))
    r["gemm_ms_each_on_compute_stream"] = gc.time_algo(algo, streams[0], reps=4) / gc.chain
    if census:
        r.update(census)
    print(json.dumps(r))
    return 0


SWEEP = [
    # (case, stream-K grid for the GEMM or None = the library's 256)
    ({"form": "packs", "k": 0, "algo": 0, "tuning": "default"}, None),
    ({"form": "gather", "k": 0, "algo": 0, "tuning": "default"}, None),
    ({"form": "fused_unpack", "k": 0, "algo": 0, "tuning": "default"}, None),
    ({"form": "packs", "k": 0, "algo": "share", "tuning": "default"}, None),
    ({"form": "packs", "k": 0, "algo": "share", "tuning": "beside"}, None),
    ({"form": "fused_unpack", "k": 0, "algo": "share", "tuning": "beside"}, None),
    ({"form": "packs", "k": 0, "algo": 0, "tuning": "beside"}, None),
    # two-sided partition: k compute units of every XCD for the sync stream, the rest for compute
    ({"form": "gather", "k": 1, "algo": 0}, None),
    ({"form": "gather", "k": 1, "algo": 0}, 248),
    ({"form": "gather", "k": 1, "algo": 0}, 224),
    ({"form": "gather", "k": 2, "algo": 0}, 224),
    ({"form": "gather", "k": 4, "algo": 0}, 224),
    ({"form": "packs", "k": 4, "algo": 0}, 224),
    ({"form": "packs", "k": 8, "algo": 0}, 192),
    ({"form": "gather", "k": 8, "algo": 0}, 192),
    ({"form": "gather", "k": 16, "algo": 0}, 128),
    # one-sided: only the sync stream is restricted
    ({"form": "gather", "k": 4, "algo": 0, "one_sided": True}, None),
]


def crossover_sweep(T):
    ref = {}        # per sync form: (T_comp, T_serial) of the unrestricted run with the library's GEMM
    for spec, grid in SWEEP:
        env = dict(os.environ)
        env.pop("TENSILE_STREAMK_FIXED_GRID", None)
        if grid:
            env["TENSILE_STREAMK_FIXED_GRID"] = str(grid)
        spec = dict(spec, T=T)
        p = subprocess.run([sys.executable, os.path.abspath(__file__), "--crossover-case", json.dumps(spec)],
                           env=env, capture_output=True, text=True, timeout=600)
        line = [ln for ln in p.stdout.splitlines() if ln.startswith("{")]
        if p.returncode != 0 or not line:
            print(json.dumps({"case": spec, "grid": grid, "failed": p.returncode, "stderr": p.stderr[-400:]}), flush=True)
            return 1
        r = json.loads(line[-1])
        form = spec.get("form", "packs")
        if not spec.get("k") and spec.get("algo") == 0 and spec.get("tuning") == "default":
            ref[form] = (r["t_comp_ms"], r["t_serial_ms"])
        r.pop("hidden_fraction_vs_unrestricted_compute", None)    # a fixed grid also binds the child's reference
        if form in ref:
            # the strict figure: every case against the computation on an unrestricted stream
            # with the library's own GEMM launch, and against that form's serial schedule
            r["t_comp_unrestricted_ms"] = ref[form][0]
            r["hidden_fraction_vs_unrestricted_compute"] = \
                1.0 - (r["t_cross_ms"] - ref[form][0]) / (ref[form][1] - ref[form][0])
        print(json.dumps({k: r.get(k) for k in (
            "case", "gemm_algorithm_index", "gemm_workgroups_per_launch", "gemm_ms_each_on_compute_stream",
            "sync_stream_compute_units", "compute_stream_compute_units", "t_comp_ms", "t_comp_unrestricted_ms",
            "t_serial_ms", "t_cross_ms", "sync_alone_ms", "end_to_end_hidden_fraction",
            "hidden_fraction_vs_unrestricted_compute", "speedup_vs_serial")}), flush=True)
    return 0


def power_probe():
    """Board power (hwmon, sampled every millisecond by a host thread) and a clock proxy (the
    duration of a fixed arithmetic-only kernel on a second stream) while the GEMM chain, the
    fused reduce + SGD, the packs, or GEMM chain and synchronisation together keep the GPU busy."""
    import glob
    import threading
    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); bs.lib(); torch.cuda.set_device(0); torch.zeros(1, device="cuda")
    files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + \
        glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
    caps = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
    cap_w = int(open(caps[0]).read()) / 1e6 if caps else None
    sclk_files = glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")    # the line marked * is the current clock

    def read_sclk():
        for ln in open(sclk_files[0]).read().splitlines():
            if ln.rstrip().endswith("*"):
                return float(ln.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        return None

    class Sampler:
        def __enter__(self):
            self.samples, self.stop = [], False
            self.t = threading.Thread(target=self.loop); self.t.start()
            return self

        def loop(self):
            self.clocks = []
            while not self.stop:
                try:
                    self.samples.append(max(int(open(f).read()) for f in files) / 1e6)
                    if sclk_files and len(self.samples) % 8 == 0:
                        c = read_sclk()
                        if c:
                            self.clocks.append(c)
                except Exception:
                    pass
                time.sleep(0.001)

        def __exit__(self, *a):
            self.stop = True; self.t.join()

        def stats(self):
            s = sorted(self.samples)
            if not s:
                return None
            c = sorted(self.clocks)
            return {"avg_W": sum(s) / len(s), "median_W": s[len(s) // 2], "max_W": s[-1], "samples": len(s),
                    "median_sclk_MHz": c[len(c) // 2] if c else None, "min_sclk_MHz": c[0] if c else None,
                    "max_sclk_MHz": c[-1] if c else None, "clock_samples": len(c)}

    gc = GemmChain()
    tb = harness.make_task(wl.VGG16, "cuda"); w = wl.VGG16
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    sink = torch.zeros(256, device="cuda")
    app = tb.make_app()

    def bg_gemm():
        gc.fn(0)(s1.cuda_stream)

    nan_y = torch.full_like(gc.Y_init, float("nan"))

    def bg_gemm_nan():          # the same GEMMs on operands that toggle no bits
        gc.enqueue(0, s1.cuda_stream, source=nan_y)

    def bg_reduce():
        for _ in range(8):
            xs.fused_reduce_sgd(tb.buckets, tb.n_bucket, tb.params, tb.momentum, w.lr, w.momentum, w.weight_decay, 1.0, stream=s1)

    def bg_packs():
        for _ in range(6):
            xs.fuse_pack_many(tb.gplan, tb.grad_tables, tb.buckets, None, s1)

    def bg_sync():
        for _ in range(4):
            app.sync(s1)

    def bg_both():
        gc.fn(0)(s1.cuda_stream)
        for _ in range(4):
            app.sync(s3)

    def measure(name, background, with_alu, seconds=1.5):
        alu_ms, bg_ms = [], []
        with Sampler() as p:
            t0 = time.time()
            while time.time() - t0 < seconds:
                t1 = time.perf_counter()
                if with_alu:            # first, so that its 256 workgroups land one per compute unit
                    a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
                    a.record(s2); bs.alu(256, 400000, sink, s2); b.record(s2)
                if background:
                    background()
                torch.cuda.synchronize()
                bg_ms.append((time.perf_counter() - t1) * 1e3)
                if with_alu:
                    alu_ms.append(a.elapsed_time(b))
        print(json.dumps({"busy_with": name, "power": p.stats(), "power_cap_W": cap_w,
                          "ms_per_round_of_that_work": _median(bg_ms),
                          "fixed_arithmetic_kernel_ms": _median(alu_ms) if alu_ms else None}), flush=True)

    measure("idle (arithmetic kernel alone)", None, True)
    measure("bf16 GEMM chain (16 GEMMs per round)", bg_gemm, False)
    measure("the same GEMM chain on NaN operands", bg_gemm_nan, False)
    measure("fused reduce+SGD, vgg16", bg_reduce, False)
    measure("fused reduce+SGD, vgg16 + arithmetic kernel", bg_reduce, True)
    measure("8 packs per launch, vgg16", bg_packs, False)
    measure("8 packs per launch, vgg16 + arithmetic kernel", bg_packs, True)
    measure("whole synchronisations, vgg16", bg_sync, False)
    measure("GEMM chain and whole synchronisations on two streams", bg_both, False)
    app.destroy()
    return 0


def footprint_probe():
    """Which neighbours does a GEMM workgroup admit on its compute unit?  For the first
    hipBLASLt algorithms: chain time alone, and the largest register footprint of a 4-wave
    workgroup (82 KiB LDS reservation) that is still placed while the GEMMs run."""
    import torch
    import bench_standin as bs
    bs.lib(); torch.cuda.set_device(0); torch.zeros(1, device="cuda")
    gc = GemmChain()
    cs, ss = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        gc.time_algo(0, cs)
    for algo in range(gc.gemm.n_algos):
        ms = gc.time_algo(algo, cs)
        fits = [v for v in (24, 48, 64, 72, 96, 128, 192, 256) if gc.admits_neighbours(algo, cs, ss, v)]
        print(json.dumps({"gemm_algorithm_index": algo, "chain_ms": ms, "gemm_ms_each": ms / gc.chain,
                          "largest_neighbour_registers_per_lane": max(fits) if fits else 0}), flush=True)
    return 0


# --------------------------------------------------------------------------- CPU baseline
def cpu_baseline(w, budget_s=8.0):
    """The oracle as it stands, like for like with `roofline`: its single-precision
    reduce + SGD alone (the arithmetic the GPU kernel performs) on a slice of the same
    buckets, one thread as written and under OpenMP on every host core the process may use.
    A second entry keeps the oracle's whole step (packs, double-precision reduce + SGD, unpack)."""
    import numpy as np
    import oracle
    from paper_2103_07974_amd import harness, workloads as wl
    cores = len(os.sched_getaffinity(0))
    n = min(w.n_elems, 32 * 1024 * 1024)
    np_dt = {"f32": np.float32, "f16": np.float16}[w.grad_dtype]
    reps = [wl.make_flat(n, w.grad_std, w.seed + 1 + r).numpy().astype(np_dt) for r in range(w.W)]
    x0 = wl.make_flat(n, w.param_std, w.seed).numpy(); v0 = wl.make_flat(n, 0.01, w.seed + 77).numpy()
    lr, mu, wd = (np.float32(w.lr).item(), np.float32(w.momentum).item(), np.float32(w.weight_decay).item())
    nbytes = (w.W * w.grad_bytes + 16) * n

    def run(threads, budget):
        x, v = x0.copy(), v0.copy()
        ts = []
        while len(ts) < 2 or (sum(ts) < budget and len(ts) < 40):
            t0 = time.perf_counter()
            oracle.reduce_sgd_f32(reps, x, v, lr, mu, wd, 1.0 / w.loss_scale, threads=threads)
            ts.append(time.perf_counter() - t0)
        return len(ts), _median(ts) * 1e3

    n1, ms1 = run(1, budget_s)
    nn, msn = run(cores, budget_s / 2)
    out = {"value": nbytes / ms1 / 1e6, "unit": "GB/s", "cores": 1, "kind": "oracle",
           "precision": "f32 (xo_reduce_sgd_f32: every operation rounded to single, as the GPU kernel)",
           "ms_per_launch": ms1,
           "sample": f"{n1} passes of the oracle's reduce + SGD over the first {n} of {w.n_elems} elements of the "
                     f"{w.name} buckets (W={w.W}, {nbytes / 1e9:.2f} GB per pass by the roofline's byte formula), "
                     f"single thread; {cores} host cores available",
           "all_cores": {"value": nbytes / msn / 1e6, "unit": "GB/s", "cores": cores, "ms_per_launch": msn,
                         "sample": f"{nn} of the same passes with the element loop under OpenMP on {cores} threads"}}
    # whole step of the oracle (its definition: double precision) on the ResNet-50-shaped set
    ws = wl.RESNET50
    grads = [[t.numpy() for t in wl.make_replica_grads(ws, r)] for r in range(ws.W)]
    params = [t.numpy() for t in wl.make_params(ws)]
    offs = oracle.layout(ws.numel, harness.DEFAULT_ALIGN)
    v = np.zeros(int(offs[-1]))
    ts = []
    while len(ts) < 2 or (sum(ts) < budget_s / 2 and len(ts) < 10):
        t0 = time.perf_counter()
        params, _ = oracle.sync_step(grads, params, v, lr, mu, wd, 1.0, align=harness.DEFAULT_ALIGN, threads=1)
        params = [p.astype(np.float32) for p in params]
        ts.append(time.perf_counter() - t0)
    sb = (ws.W * ws.grad_bytes + 16) * ws.n_elems
    out["whole_step"] = {"value": sb / (_median(ts) * 1e3) / 1e6, "unit": "GB/s", "cores": 1,
                         "precision": "f64 (xo_reduce_sgd_f64, the definition)", "ms_per_step": _median(ts) * 1e3,
                         "sample": f"{len(ts)} whole {ws.name} steps (W={ws.W} packs, reduce + SGD, unpack), single thread"}
    return out


# --------------------------------------------------------------------------- profiling modes
def kernels_only(name, launches, pooled=True):
    """Stand-alone launches of every kernel of one workload and nothing else, for
    `rocprofv3 --kernel-trace --stats`: each kernel's average is then its stand-alone time."""
    import torch
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); torch.cuda.set_device(0)
    w = wl.WORKLOADS[name]
    n_sets = 3 if name == "resnet50" else 1
    tasks = [harness.make_task(w, "cuda", pooled=pooled) for _ in range(n_sets)]
    for t in tasks:
        t.momentum.copy_(wl.make_flat(t.n_bucket, 0.01, w.seed + 77, device="cuda"))
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for i in range(launches):
            t = tasks[i % n_sets]
            xs.fuse_pack_many(t.gplan, t.grad_tables, t.buckets, None, s)
        for i in range(launches):
            t = tasks[i % n_sets]
            xs.fused_reduce_sgd(t.buckets, t.n_bucket, t.params, t.momentum, w.lr, w.momentum, w.weight_decay,
                                1.0 / w.loss_scale, stream=s)
        for i in range(launches):
            t = tasks[i % n_sets]
            xs.fuse_unpack(t.pplan, t.params, t.param_table, s)
        for i in range(launches):
            t = tasks[i % n_sets]
            xs.fused_reduce_sgd_unpack(t.gplan, t.buckets, t.params, t.momentum, t.param_table, w.lr, w.momentum,
                                       w.weight_decay, 1.0 / w.loss_scale, stream=s)
        for i in range(launches):
            t = tasks[i % n_sets]
            xs.fused_gather_reduce_sgd(t.gplan, t.gather_table, w.W, t.params, t.momentum, w.lr, w.momentum,
                                       w.weight_decay, 1.0 / w.loss_scale, param_tensor_ptrs=t.param_table, stream=s)
        torch.cuda.synchronize()
    t = tasks[0]
    print(json.dumps({"workload": name, "launches_of_each_kernel": launches, "W": w.W, "elements": w.n_elems,
                      "bytes": {"pack_all_replicas": w.W * t.pack_bytes(), "reduce_sgd": t.reduce_bytes(),
                                "unpack": t.unpack_bytes(), "reduce_sgd_fused_unpack": t.reduce_bytes() + 4 * w.n_elems,
                                "gather_form": t.gather_bytes(True)}}))
    return 0


def traffic_probe(name, pooled=True):
    """A few launches for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`, one workload per
    process: a plain device copy of known size first (its counter reading calibrates the
    unit), then every kernel of the path.  Nothing is freed while the counters are collected
    (the first version of this probe released its buffers between workloads inside one
    profiled process and that process ended in a host-side segmentation fault inside the
    profiling layer at the next allocation)."""
    import torch
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib()
    torch.cuda.set_device(0)
    n = 256 * 1024 * 1024                       # 1 GiB read + 1 GiB written per copy
    src = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    w = wl.WORKLOADS[name]
    # the largest set: all workers' tensor lists point at worker 0's tensors (the buckets stay
    # distinct), which keeps the number of set-up launches under the counters small
    task = harness.make_task(w, "cuda", shared_grads=name == "bert_large_f16", pooled=pooled)
    for _ in range(3):
        xs.fuse_pack(task.gplan, task.grad_tables[0], task.buckets[0])
        xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
        xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum,
                            w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale)
        xs.fuse_unpack(task.pplan, task.params, task.param_table)
        xs.fused_reduce_sgd_unpack(task.gplan, task.buckets, task.params, task.momentum, task.param_table,
                                   w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale)
        xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, task.params,
                                   task.momentum, w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale,
                                   param_tensor_ptrs=task.param_table)
    torch.cuda.synchronize()
    print(json.dumps({"workload": w.name, "copy_bytes_each_way": n * 4, "W": w.W,
                      "reduce_bytes": task.reduce_bytes(), "pack_bytes_one_replica": task.pack_bytes(),
                      "unpack_bytes": task.unpack_bytes(), "gather_bytes": task.gather_bytes(True),
                      "reduce_fused_unpack_bytes": task.reduce_bytes() + 4 * w.n_elems,
                      "bucket_elems": task.n_bucket}))
    return 0


def stream_ceiling():
    """Attainable HBM rate of plain streaming kernels with the access mix of pack/unpack (1:1
    copy) and of the fused reduce + SGD at W = 8 (10 streams read, 2 written): one-wavefront
    workgroups in address order, one 16-byte vector per lane, non-temporal accesses, random
    data, buffers of the VGG-16 bucket's size carved from one allocation as the harness lays a
    task out, for several occupancy caps (LDS reserved per workgroup)."""
    import torch
    import bench_standin as bs
    bs.lib(); torch.cuda.set_device(0)
    s = torch.cuda.Stream()
    from paper_2103_07974_amd import xs
    n = 138357568                              # elements per buffer: the VGG-16-shaped bucket
    bufs = [b.normal_(0, 1e-3) for b in xs.pool_alloc([(n, torch.float32)] * 12)]   # one allocation, as the
                                                                                   # harness lays a task out
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for lds in (0, 8192, 16384, 32768):
        ms = _median(timed_launches(lambda i: bs.copy(bufs[i % 5], bufs[5 + i % 5], lds, s), s, 30, 5))
        print(json.dumps({"kernel": "copy 1 read : 1 write", "lds_reserve": lds, "ms": ms, "GBs": 2 * n * 4 / ms / 1e6}), flush=True)
        ms = _median(timed_launches(lambda i: bs.mix(bufs[:10], bufs[10], bufs[11], lds, s), s, 30, 5))
        print(json.dumps({"kernel": "10 reads : 2 writes", "lds_reserve": lds, "ms": ms, "GBs": 12 * n * 4 / ms / 1e6}), flush=True)
        ms = _median(timed_launches(lambda i: bs.read(bufs[:10], sink, lds, s), s, 30, 5))
        print(json.dumps({"kernel": "10 reads, no write", "lds_reserve": lds, "ms": ms, "GBs": 10 * n * 4 / ms / 1e6}), flush=True)
    return 0


def few_cu_sweep():
    """The VGG-16-shaped synchronisation alone on a stream that owns k compute units of every
    XCD, for several launch shapes: what a synchronisation confined to few compute units can
    move, per compute unit and in all."""
    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); bs.lib(); torch.cuda.set_device(0); torch.zeros(1, device="cuda")
    w = wl.VGG16
    tb = harness.make_task(w, "cuda")

    def tuned(**kw):
        t = xs.tuning_preset(xs.PRESET_ALONE)
        for name, v in kw.items():
            t[getattr(xs, "TUNE_" + name)] = v
        return t
    shapes = [
        ("default: one row per one-wave workgroup, 13 resident per CU", tuned()),
        ("20 resident per CU", tuned(GATHER_LDS_RESERVE=8192)),
        ("10 resident per CU", tuned(GATHER_LDS_RESERVE=16384)),
        ("as many as the registers allow", tuned(GATHER_LDS_RESERVE=0)),
        ("persistent grid, 10 one-wave workgroups per CU of the chip", tuned(REDUCE_WG_PER_CU=10, GATHER_LDS_RESERVE=0)),
        ("4-wave workgroups, 5 resident per CU", tuned(REDUCE_WAVES_PER_WG=4, GATHER_LDS_RESERVE=32768)),
    ]
    nbytes = tb.gather_bytes()
    for k in (1, 2, 4, 8, 32):
        if k == 32:
            stream, n_cus, ms = torch.cuda.Stream(), 256, None
        else:
            ms = bs.MaskedStream(bs.sync_and_compute_masks(k)[0])
            stream, n_cus = ms.stream, len(bs.census(4096, 2000, ms.stream))
        for label, tn in shapes:
            app = tb.make_app(None, tuning=tn, fused_gather=True)
            for _ in range(2):
                app.sync(stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n = 3 if k < 4 else 10
            for _ in range(n):
                app.sync(stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e3 / n
            app.destroy()
            print(json.dumps({"compute_units": n_cus, "launch": label, "sync_ms": dt, "GBs": nbytes / dt / 1e6,
                              "GBs_per_compute_unit": nbytes / dt / 1e6 / n_cus}), flush=True)
    return 0


def ratio_sweep():
    """Section 1, first contribution: the synchronisation delay disappears while comm/comp < 1.
    The pair of config 4 (ResNet-50- and VGG-16-shaped synchronisations, gathering form) beside
    an arithmetic-only computation of varied length, i.e. at varied comm/comp ratio, against
    the timeline model of Algorithm 1 for two tasks: one outer iteration lasts
    max(C_A, M_B) + max(C_B, M_A)."""
    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); bs.lib(); torch.cuda.set_device(0); torch.zeros(1, device="cuda")
    pair = [harness.make_task(wl.RESNET50, "cuda"), harness.make_task(wl.VGG16, "cuda")]
    cs, ss = torch.cuda.Stream(), torch.cuda.Stream()
    for target_ms in (0.3, 0.6, 0.9, 1.2, 1.8, 2.4, 4.8, 9.6):
        alu, label = alu_standin(target_ms)
        r = crossover_run(pair, [alu, alu], label, T=20, rounds=3, form="gather", streams=(cs, ss))
        C, M = r["compute_alone_ms"], r["sync_alone_ms"]
        model_extra = max(0.0, M[1] - C[0]) + max(0.0, M[0] - C[1])        # per outer iteration
        print(json.dumps({
            "compute_ms": C, "sync_alone_ms": M, "comm_comp_ratio_task_B": M[1] / C[0], "comm_comp_ratio_task_A": M[0] / C[1],
            "hidden_fraction_measured": r["end_to_end_hidden_fraction"],
            "hidden_fraction_timeline_model": 1.0 - model_extra / (M[0] + M[1]),
            "t_comp_ms": r["t_comp_ms"], "t_serial_ms": r["t_serial_ms"], "t_cross_ms": r["t_cross_ms"],
            "t_cross_timeline_model_ms": r["T"] * (max(C[0], M[1]) + max(C[1], M[0])) + M[1],
            "per_task_hidden": [p["hidden_fraction"] for p in r.get("per_task", [])]}), flush=True)
    return 0


# --------------------------------------------------------------------------- main
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--quick", action="store_true", help="headline workload and rooflines only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--T", type=int, default=20, help="outer iterations of the crossover schedule")
    ap.add_argument("--kernels-only", metavar="WORKLOAD", help="resnet50 | vgg16 | bert_large_f16")
    ap.add_argument("--launches", type=int, default=60)
    ap.add_argument("--traffic-probe", metavar="WORKLOAD", help="resnet50 | vgg16 | bert_large_f16")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="with --traffic-probe / --kernels-only: every bucket, parameters and momentum in an "
                         "allocation of their own instead of one pool")
    ap.add_argument("--stream-ceiling", action="store_true")
    ap.add_argument("--power", action="store_true")
    ap.add_argument("--footprint", action="store_true")
    ap.add_argument("--few-cu-sweep", action="store_true")
    ap.add_argument("--ratio-sweep", action="store_true")
    ap.add_argument("--crossover-sweep", action="store_true")
    ap.add_argument("--crossover-case", metavar="JSON")
    ap.add_argument("--crossover-only", action="store_true",
                    help="one short two-stream run (for rocprofv3 --kernel-trace); with --form, --share, --beside")
    ap.add_argument("--form", default="packs", choices=["packs", "gather", "fused_unpack"])
    ap.add_argument("--share", action="store_true", help="GEMM algorithm that leaves room for neighbours")
    ap.add_argument("--share-tolerance", type=float, default=1.10,
                    help="how much slower than the fastest GEMM algorithm the sharing one may be")
    ap.add_argument("--beside", action="store_true", help="XS_PRESET_BESIDE_COMPUTE for the synchronisations")
    ap.add_argument("--autograd", action="store_true", help="with --crossover-only: the two autograd MLP tasks")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="with --crossover-only: one launch setting of the synchronisations, by the name of its "
                         "key without the XS_TUNE_ prefix (e.g. REDUCE_WG_PER_CU=2); may be repeated")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the W workers' gradients are resident "
              "on that GPU); --gpus must be 1", file=sys.stderr)
        return 2
    if args.crossover_sweep:           # the parent never touches the GPU: one child per case
        return crossover_sweep(min(args.T, 10))
    if args.crossover_case:
        return crossover_case(json.loads(args.crossover_case))
    if args.kernels_only:
        return kernels_only(args.kernels_only, args.launches, not args.separate_allocations)
    if args.traffic_probe:
        return traffic_probe(args.traffic_probe, not args.separate_allocations)
    if args.stream_ceiling:
        return stream_ceiling()
    if args.power:
        return power_probe()
    if args.footprint:
        return footprint_probe()
    if args.few_cu_sweep:
        return few_cu_sweep()
    if args.ratio_sweep:
        return ratio_sweep()

    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib(); bs.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    if args.crossover_only:
        cs, ss = torch.cuda.Stream(), torch.cuda.Stream()
        tuning = xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE) if args.beside else None
        if args.tune:
            tuning = tuning if tuning is not None else xs.tuning_preset(xs.PRESET_ALONE)
            for item in args.tune:
                name, _, value = item.partition("=")
                tuning[getattr(xs, "TUNE_" + name)] = int(value)
        if args.autograd:
            ma = harness.make_mlp_task("mlp_6x4096", [4096] * 7, W=4, batch=256, seed=31)
            mb = harness.make_mlp_task("mlp_8192_wide", [2048, 8192, 8192, 2048], W=4, batch=256, seed=32)
            r = crossover_run([ma.state, mb.state], [ma.compute, mb.compute], "autograd forward+backward of two fp32 MLPs",
                              T=args.T, form=args.form, tuning=tuning, streams=(cs, ss), cross_only=True)
        else:
            gc = GemmChain()
            algo = gc.choose_for_sharing(cs, ss, args.share_tolerance)[0] if args.share else 0
            ta = harness.make_task(wl.RESNET50, "cuda"); tb = harness.make_task(wl.VGG16, "cuda")
            r = crossover_run([ta, tb], [gc.fn(algo)] * 2, gc.label, T=args.T, form=args.form, tuning=tuning,
                              streams=(cs, ss), cross_only=True)
            r["gemm_algorithm_index"] = algo
        print(json.dumps(r))
        return 0

    # ---- headline: whole steps of the VGG-16-shaped set ------------------------------------
    w = wl.VGG16
    vgg = harness.make_task(w, "cuda")
    vgg.momentum.copy_(wl.make_flat(vgg.n_bucket, 0.01, w.seed + 77, device="cuda"))   # steady state
    ms_per_step, kernel_ms = time_steps([vgg], args.steps, args.warmup, stream)
    reduce_bytes = vgg.reduce_bytes()
    st = _stats(kernel_ms)
    achieved = reduce_bytes / st["avg_launch_ms"] / 1e6
    out = {
        "metric": METRIC, "value": reduce_bytes / ms_per_step / 1e6, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "vgg16-shaped gradient set, 32 tensors, 138,357,544 elements, W=8 fp32 replicas; "
                               "step = 8 packs (one launch) + fused reduce+SGD + unpack on one stream",
                   "W": w.W, "n_elems": w.n_elems, "n_tensors": w.n_tensors, "bucket_align_elems": vgg.align,
                   "bytes_per_step_counted": reduce_bytes},
        "roofline": {"bound": "hbm", "kernel": "xs::reduce_sgd_kernel<8, 0, false, true, true, false, false>",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_launch": reduce_bytes, "bytes_per_element": 48,
                     "timed": "HIP events on the launch stream around every reduce + SGD launch of the timed steps", **st},
        "from_profiles": FROM_PROFILES,
    }
    ms_fused, _ = time_steps([vgg], max(10, args.steps // 2), 5, stream, fused_unpack=True)
    extra = {"vgg16": {"step_ms": ms_per_step, "step_with_fused_unpack_ms": ms_fused,
                       "step_with_fused_unpack_GBs_by_headline_formula": reduce_bytes / ms_fused / 1e6}}
    by_config = {"vgg16": reduce_roofline([vgg], stream, 50, 10)}
    extra["vgg16"].update(other_kernels([vgg], stream))

    # ---- the other bar configs, stand-alone ------------------------------------------------
    rn = [harness.make_task(wl.RESNET50, "cuda") for _ in range(3)]      # three sets: 204 MB of state
    for t in rn:                                                       # would nearly fit the 256 MB cache
        t.momentum.copy_(wl.make_flat(t.n_bucket, 0.01, wl.RESNET50.seed + 77, device="cuda"))
    by_config["resnet50"] = reduce_roofline(rn, stream, 60, 12)
    ms_rn, _ = time_steps(rn, 60, 12, stream)
    ms_rn_fused, _ = time_steps(rn, 60, 12, stream, fused_unpack=True)
    extra["resnet50"] = {"step_ms": ms_rn, "step_with_fused_unpack_ms": ms_rn_fused,
                         "step_GBs_by_headline_formula": rn[0].reduce_bytes() / ms_rn / 1e6,
                         "buffer_sets_rotated": 3}
    if not args.quick:
        extra["resnet50"].update(other_kernels(rn, stream))
    resnet = rn[0]
    del rn
    torch.cuda.empty_cache()
    bert = harness.make_task(wl.BERT_LARGE_F16, "cuda")
    bert.momentum.copy_(wl.make_flat(bert.n_bucket, 0.01, wl.BERT_LARGE_F16.seed + 77, device="cuda"))
    by_config["bert_large_f16"] = reduce_roofline([bert], stream, 50, 10)
    if not args.quick:
        extra["bert_large_f16"] = other_kernels([bert], stream, launches=12, warmup=3)
        extra["bert_large_f16"]["overflow_skip"] = time_overflow_skip(bert, stream)
    del bert
    torch.cuda.empty_cache()
    out["roofline_by_config"] = by_config

    if not args.quick:
        # ---- launch-bound end: the tiny set -------------------------------------------------
        tiny = harness.make_task(wl.TINY_MLP, "cuda")
        tk = {}
        for form, key in (("packs", "step_latency_us"), ("fused_unpack", "fused_unpack_step_latency_us"),
                          ("gather", "gather_step_latency_us")):
            app = tiny.make_app(fused_gather=form == "gather", fused_unpack=form == "fused_unpack")
            with torch.cuda.stream(stream):
                for _ in range(20):
                    app.sync(stream)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(200):
                    app.sync(stream)
                torch.cuda.synchronize()
                tk[key] = (time.perf_counter() - t0) * 1e6 / 200
            if form == "gather":        # the same step replayed from a captured HIP graph of ten
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for _ in range(10):
                        app.sync(stream)
                for _ in range(3):
                    graph.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(20):
                    graph.replay()
                torch.cuda.synchronize()
                tk["gather_step_latency_graph_us"] = (time.perf_counter() - t0) * 1e6 / 200
                del graph
            app.destroy()
        extra["tiny_mlp"] = tk

        # ---- crossover (config 4) ------------------------------------------------------------
        cs, ss = torch.cuda.Stream(), torch.cuda.Stream()       # one pair of streams for every run
        gc = GemmChain()
        for _ in range(3):                                      # brings the chip to its loaded state
            gc.time_algo(0, cs)
        share_algo, algo_ms = gc.choose_for_sharing(cs, ss, 1.10)
        beside = xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE)
        pair = [resnet, vgg]
        f0, fs = gc.fn(0), gc.fn(share_algo)
        x = {}
        x["packs_form"] = crossover_run(pair, [f0, f0], gc.label, T=args.T, form="packs", streams=(cs, ss))
        x["gather_form"] = crossover_run(pair, [f0, f0], gc.label, T=args.T, form="gather", streams=(cs, ss))
        x["fused_unpack_form"] = crossover_run(pair, [f0, f0], gc.label, T=args.T, form="fused_unpack", streams=(cs, ss))
        T2 = max(4, args.T // 2)      # the variants beside config 4 proper run half as many iterations
        ref = x["packs_form"]["t_comp_ms"] * T2 / args.T
        x["packs_form_sharing_gemm_kernel"] = crossover_run(pair, [fs, fs], gc.label, T=T2, form="packs", streams=(cs, ss),
                                                            t_comp_reference=ref)
        x["packs_form_sharing_gemm_kernel_beside_preset"] = crossover_run(
            pair, [fs, fs], gc.label, T=T2, form="packs", tuning=beside, streams=(cs, ss), t_comp_reference=ref)
        alu, alu_label = alu_standin(x["packs_form"]["compute_alone_ms"][0])
        x["alu_standin_packs_form"] = crossover_run(pair, [alu, alu], alu_label, T=T2, form="packs", streams=(cs, ss))
        # the row-per-wavefront copy kernels fill every wave slot of the chip by default; a compute
        # kernel of one long-lived workgroup per compute unit that is dispatched meanwhile lands
        # unevenly and stays so.  XS_PRESET_LEAVE_WAVE_SLOTS caps the copies at 10 per compute unit.
        x["alu_standin_packs_form_leave_wave_slots_preset"] = crossover_run(
            pair, [alu, alu], alu_label, T=T2, form="packs",
            tuning=xs.tuning_preset(xs.PRESET_LEAVE_WAVE_SLOTS), streams=(cs, ss))
        x["alu_standin_gather_form"] = crossover_run(pair, [alu, alu], alu_label, T=T2, form="gather", streams=(cs, ss))
        # N = 3 tasks (Algorithm 1 is written for N): a second ResNet-50-shaped task joins
        third = harness.make_task(wl.RESNET50, "cuda")
        x["n3_packs_form"] = crossover_run([resnet, vgg, third], [f0, f0, f0], gc.label, T=max(4, T2 // 2),
                                           form="packs", streams=(cs, ss))
        x["n3_alu_standin_gather_form"] = crossover_run([resnet, vgg, third], [alu, alu, alu], alu_label,
                                                        T=max(4, T2 // 2), form="gather", streams=(cs, ss))
        del third
        # every case against the computation with the library's own GEMM kernel (a slower GEMM
        # that shares its compute units must make up for its own slowness first)
        def strict(k):
            v = x[k].get("hidden_fraction_vs_unrestricted_compute")
            return x[k]["end_to_end_hidden_fraction"] if v is None else v
        best_key = max((k for k in x if "alu" not in k and "n3" not in k and x[k].get("end_to_end_hidden_fraction") is not None),
                       key=strict)
        x["gemm_chain_ms_by_algorithm"] = {str(a): t for a, t in algo_ms.items()}
        x["gemm_algorithm_that_admits_neighbours"] = share_algo
        extra["crossover"] = x
        del vgg, resnet, pair
        torch.cuda.empty_cache()

        # a real forward + backward (autograd, fp32 MLPs of about 100 M parameters, one
        # micro-batch per worker) as each task's computation instead of a stand-in
        ma = harness.make_mlp_task("mlp_6x4096", [4096] * 7, W=4, batch=256, seed=31)
        mb = harness.make_mlp_task("mlp_8192_wide", [2048, 8192, 8192, 2048], W=4, batch=256, seed=32)
        lab = "autograd forward+backward of fp32 ReLU MLPs (6x4096^2 / 2048-8192-8192-2048), 4 micro-batches of 256"
        x["autograd_mlp_packs_form"] = crossover_run(
            [ma.state, mb.state], [ma.compute, mb.compute], lab, T=10, form="packs", streams=(cs, ss), rounds=3)
        x["autograd_mlp_gather_form"] = crossover_run(
            [ma.state, mb.state], [ma.compute, mb.compute], lab, T=10, form="gather", streams=(cs, ss), rounds=3)
        del ma, mb
        torch.cuda.empty_cache()

        c = x["packs_form"]
        out["crossover"] = {
            "config": "ResNet-50-shaped (A) and VGG-16-shaped (B) synchronisations beside " + c["compute"] + f", T={c['T']}",
            "definition": "1 - (T_cross - T_comp) / (T_serial - T_comp), medians of interleaved rounds",
            "end_to_end_hidden_fraction": c["end_to_end_hidden_fraction"],
            "target": 0.90,
            "target_met": bool(c["end_to_end_hidden_fraction"] is not None and c["end_to_end_hidden_fraction"] >= 0.90),
            "speedup_vs_serial": c["speedup_vs_serial"],
            "per_task": {"A_resnet50": c["per_task"][0], "B_vgg16": c["per_task"][1]},
            "best_of_the_library_s_forms_and_settings": {"which": best_key, "end_to_end_hidden_fraction": strict(best_key)},
            "why": "the bf16 GEMM chain alone runs at the board's 1400 W power limit (shader clock 1.9 of 2.4 GHz) and its kernel owns every "
                   "compute unit whole; the HBM-bound synchronisation kernels draw 1.0-1.2 kW themselves, so what "
                   "runs beside the GEMMs is paid back in GEMM time, and every partition of the compute units costs "
                   "the GEMM more than the synchronisations take "
                   "(profiles/crossover_config4_partition_sweep_and_power.md)",
            "other_figures_that_are_not_the_target_metric": {
                "iterations_whose_sync_outlasted_the_compute_beside_it": c["iterations_whose_sync_outlasted_the_compute_beside_it"],
                "of_iterations": c["of_iterations"],
                "end_to_end_hidden_fraction_beside_an_arithmetic_only_standin": x["alu_standin_gather_form"]["end_to_end_hidden_fraction"],
                "end_to_end_hidden_fraction_n3": x["n3_packs_form"]["end_to_end_hidden_fraction"]},
        }
    out["extra"] = extra
    out["cpu_baseline"] = None if args.no_cpu else cpu_baseline(w)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
