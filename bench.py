#!/usr/bin/env python3
"""Benchmark of the fused gradient-synchronisation path on one MI355X.

A step is one whole synchronisation of the ResNet-50-shaped gradient set: the W = 8 packs
(one launch), the fused reduce + SGD, and the unpack of the parameters, on one stream, inputs
resident in HBM.  `value` is (W*s + 16) * N bytes (W replica buckets, parameters and momentum read,
parameters and momentum written) divided by the time of the whole step.  `roofline`
covers the fused reduce + SGD kernel alone, timed with events inside the timed region.
The VGG-16- and BERT-large-shaped sets, the tiny set's latency and the two-stream
crossover pair are measured after the timed region and reported under `extra`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the fused reduce + SGD kernel on the headline workload, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a plain copy's reading of the same
# counters (profiles/hbm_traffic_pmc_reduce_sgd_pack_unpack.md)
MEASURED_TRAFFIC_BYTES = 1226785792
# share of the sync kernels' time that lies inside the other task's compute kernels in the
# crossover config, from the rocprofv3 kernel trace
# (profiles/crossover_kernel_trace_resnet50_vgg16_gemm_chain.md)
STREAM_OVERLAP_FROM_TRACE = 0.983


def _median(xs_):
    s = sorted(xs_)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def time_steps(tasks, steps, warmup, stream):
    """K whole steps, rotating over independent buffer sets so that no step finds its
    state in the 256 MB last-level cache; events around the reduce kernel of each step."""
    import torch
    from paper_2103_07974_amd import xs
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]

    def one(task, pair=None):
        w = task.workload
        xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets, None, stream)
        if pair:
            pair[0].record(stream)
        xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum,
                            w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale, stream=stream)
        if pair:
            pair[1].record(stream)
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
    kernel_ms = [a.elapsed_time(b) for a, b in ev]
    return (t1 - t0) * 1e3 / steps, kernel_ms


def time_kernels(task, stream, reps=30, warm=5):
    """Per-kernel medians (ms) for pack (one replica), reduce + SGD, unpack."""
    import torch
    from paper_2103_07974_amd import xs
    w = task.workload
    out = {}

    def run(fn):
        ts = []
        with torch.cuda.stream(stream):
            for i in range(warm + reps):
                a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
                a.record(stream); fn(i); b.record(stream)
                b.synchronize()
                if i >= warm:
                    ts.append(a.elapsed_time(b))
        return ts

    out["pack_ms"] = _median(run(lambda i: xs.fuse_pack(
        task.gplan, task.grad_tables[i % w.W], task.buckets[i % w.W], None, stream)))
    out["pack_all_replicas_ms"] = _median(run(lambda i: xs.fuse_pack_many(
        task.gplan, task.grad_tables, task.buckets, None, stream)))
    out["pack_all_replicas_GBs"] = w.W * task.pack_bytes() / out["pack_all_replicas_ms"] / 1e6
    red = run(lambda i: xs.fused_reduce_sgd(
        task.buckets, task.n_bucket, task.params, task.momentum, w.lr, w.momentum,
        w.weight_decay, 1.0 / w.loss_scale, stream=stream))
    out["reduce_sgd_ms"] = _median(red)
    out["reduce_sgd_min_ms"] = min(red)
    out["unpack_ms"] = _median(run(lambda i: xs.fuse_unpack(
        task.pplan, task.params, task.param_table, stream)))
    out["reduce_sgd_GBs"] = task.reduce_bytes() / out["reduce_sgd_ms"] / 1e6
    out["reduce_sgd_frac_of_hbm_peak"] = out["reduce_sgd_GBs"] / HBM_PEAK_GBS
    out["pack_GBs"] = task.pack_bytes() / out["pack_ms"] / 1e6
    out["unpack_GBs"] = task.unpack_bytes() / out["unpack_ms"] / 1e6
    return out


def time_gather(tasks, stream, reps=30, warm=6):
    """The gathering form (no buckets, parameter views written in the same pass): one kernel
    is the whole step.  Rotates over the buffer sets like the timed region."""
    import torch
    from paper_2103_07974_amd import xs
    ts = []
    with torch.cuda.stream(stream):
        for i in range(warm + reps):
            t = tasks[i % len(tasks)]; w = t.workload
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            xs.fused_gather_reduce_sgd(t.gplan, t.gather_table, w.W, t.params, t.momentum, w.lr,
                                       w.momentum, w.weight_decay, 1.0 / w.loss_scale,
                                       param_tensor_ptrs=t.param_table, stream=stream)
            b.record(stream); b.synchronize()
            if i >= warm:
                ts.append(a.elapsed_time(b))
    ms = _median(ts)
    return {"step_ms": ms, "min_ms": min(ts),
            "GBs_moved": tasks[0].gather_bytes(True) / ms / 1e6,
            "frac_of_hbm_peak": tasks[0].gather_bytes(True) / ms / 1e6 / HBM_PEAK_GBS,
            "GBs_by_headline_formula": tasks[0].reduce_bytes() / ms / 1e6}


def time_param_groups(tasks, stream, reps=30, warm=6):
    """Both forms with one (lr, momentum, weight decay) record per tensor: weight decay on
    matrices and filters only, biases and normalisation parameters in a group of their own.
    Same bytes as the single-triple forms plus a 16-byte record per tensor."""
    import torch
    from paper_2103_07974_amd import xs
    w = tasks[0].workload
    table = xs.tensor_hparams_table([(w.lr, w.momentum, w.weight_decay) if len(s) > 1
                                     else (2 * w.lr, w.momentum, 0.0) for s in w.shapes])
    out = {}
    for form in ("bucket", "gather"):
        ts = []
        with torch.cuda.stream(stream):
            for i in range(warm + reps):
                t = tasks[i % len(tasks)]
                a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
                a.record(stream)
                if form == "bucket":
                    xs.fused_reduce_sgd_pt(t.gplan, t.buckets, t.params, t.momentum, table,
                                           1.0 / w.loss_scale, stream=stream)
                else:
                    xs.fused_gather_reduce_sgd_pt(t.gplan, t.gather_table, w.W, t.params, t.momentum,
                                                  table, 1.0 / w.loss_scale,
                                                  param_tensor_ptrs=t.param_table, stream=stream)
                b.record(stream); b.synchronize()
                if i >= warm:
                    ts.append(a.elapsed_time(b))
        ms = _median(ts)
        nbytes = tasks[0].reduce_bytes() if form == "bucket" else tasks[0].gather_bytes(True)
        out[form + "_form"] = {"ms": ms, "GBs": nbytes / ms / 1e6,
                               "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS}
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


def crossover_pair(task_a, task_b, T=20, chain=16, dim=8192, fused_gather=False, standin="gemm",
                   cross_only=False, computes=None, label=None, streams=None, tuning=None, rounds=5):
    """Two tasks alternate as in Algorithm 1: one computes (a stand-in for forward + backward)
    while the other synchronises on the second stream.

    standin="gemm": the configured chain of bf16 GEMMs.  standin="alu": one arithmetic-only
    kernel of ordinary occupancy and no memory traffic (xs_standin_alu) of the same duration -
    the kind of kernel a synchronisation wave can share a compute unit with.
    computes=(fn_a, fn_b): each task's own computation instead of a stand-in."""
    import torch
    import bench_standin as bs
    from paper_2103_07974_amd import xs
    g = torch.Generator(device="cuda"); g.manual_seed(task_a.workload.seed + 100)
    if computes is not None:
        pass
    elif standin == "gemm":
        B = (torch.randn(dim, dim, generator=g, device="cuda") / dim ** 0.5).to(torch.bfloat16)
        Y = [torch.randn(dim, dim, generator=g, device="cuda").to(torch.bfloat16) for _ in range(2)]

        def compute(stream_ptr):
            s = torch.cuda.ExternalStream(stream_ptr)
            with torch.cuda.stream(s):
                for k in range(chain):
                    torch.matmul(Y[k & 1], B, out=Y[1 - (k & 1)])
        label = f"{chain}x[{dim}x{dim}]@[{dim}x{dim}] bf16"
    else:
        # arithmetic only: one kernel of 256 workgroups of 256 lanes (one per compute unit, a
        # quarter of the wave slots, few registers, no memory traffic); iteration count
        # calibrated so that it lasts as long as the GEMM chain does
        sink = torch.zeros(256, device="cuda")
        target_ms, probe_iters = 12.6, 100000
        a0 = torch.cuda.Event(enable_timing=True); a1 = torch.cuda.Event(enable_timing=True)
        bs.alu(256, probe_iters, sink); torch.cuda.synchronize()
        a0.record(); bs.alu(256, probe_iters, sink); a1.record(); a1.synchronize()
        iters = max(1000, int(probe_iters * target_ms / a0.elapsed_time(a1)))

        def compute(stream_ptr):
            bs.alu(256, iters, sink, stream_ptr)
        label = f"one arithmetic-only kernel, 256x256 lanes, {iters} x 8 multiply-adds per lane"
    if computes is None:
        computes = (compute, compute)
    # `tuning`: launch settings of the synchronisations inside the two-stream schedule; the
    # serial schedule and the stand-alone timings always use the defaults (the fastest sync)
    apps = [task_a.make_app(computes[0], fused_gather=fused_gather, tuning=tuning),
            task_b.make_app(computes[1], fused_gather=fused_gather, tuning=tuning)]
    apps_alone = apps if tuning is None else [task_a.make_app(computes[0], fused_gather=fused_gather),
                                              task_b.make_app(computes[1], fused_gather=fused_gather)]
    cs, ss = streams if streams is not None else (torch.cuda.Stream(), torch.cuda.Stream())

    def run_cross(record=None):
        # Algorithm 1, N = 2, T outer iterations: the first inner step has nothing to
        # receive, every later one synchronises the task that computed before it, and the
        # last task's gradients are drained at the end: 2T computations, 2T synchronisations
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        xs.crossover_step(apps[0], None, cs, ss)
        for k in range(1, 2 * T):
            i = k % 2
            xs.crossover_step(apps[i], apps[1 - i], cs, ss)
            if record is not None:
                es = torch.cuda.Event(enable_timing=True); ec = torch.cuda.Event(enable_timing=True)
                es.record(ss); ec.record(cs)
                record.append((1 - i, es, ec))
        xs.crossover_drain(apps[1], ss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_serial():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(T):
            for i in (0, 1):
                computes[i](cs.cuda_stream)
                apps_alone[i].sync(cs)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_comp():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(2 * T):
            computes[t % 2](cs.cuda_stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def run_sync(app, n=10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            app.sync(ss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    if cross_only:       # for kernel tracing: nothing but the two-stream schedule itself
        run_cross()
        ms = run_cross()
        for a in apps:
            a.destroy()
        return {"T": T, "compute_standin": label, "t_cross_ms": ms,
                "sync_kernels": "gather form" if fused_gather else "packs, reduce+SGD, unpack"}
    # The chip's clocks drift with its thermal and power state (the GEMM chain runs at the
    # board's power limit), by more than the difference that is being measured; the three
    # modes are therefore run round-robin and every figure is a median over the rounds.
    run_comp(); run_serial(); run_cross(); run_comp(); run_serial(); run_cross()     # warm-up
    rec = []
    rows = []
    for r in range(rounds):
        rows.append((run_comp(), run_serial(), run_cross(rec if r == rounds - 1 else None)))
    t_comp = _median([x[0] for x in rows])
    t_serial = _median([x[1] for x in rows])
    t_cross = _median([x[2] for x in rows])
    per_round_hidden = [1.0 - (x[2] - x[0]) / (x[1] - x[0]) for x in rows if x[1] > x[0]]
    sync_a, sync_b = run_sync(apps_alone[0]), run_sync(apps_alone[1])
    sum_sync = t_serial - t_comp
    # event view: how long each synchronisation ran past the end of the computation beside it
    exposed = {0: 0.0, 1: 0.0}; count = {0: 0, 1: 0}; late = {0: 0, 1: 0}
    for who, es, ec in rec:
        d = ec.elapsed_time(es)            # > 0: the sync finished after the compute beside it
        count[who] += 1
        if d > 0:
            exposed[who] += d; late[who] += 1
    res = {
        "T": T, "compute_standin": label,
        "sync_kernels": "gather+reduce+SGD+views (1 kernel)" if fused_gather else "W packs (1 launch), reduce+SGD, unpack",
        "t_comp_ms": t_comp, "t_serial_ms": t_serial, "t_cross_ms": t_cross,
        "sum_sync_ms": sum_sync, "sync_a_alone_ms": sync_a, "sync_b_alone_ms": sync_b,
        "compute_chain_ms": t_comp / (2 * T),
        "comm_comp_ratio_a": sync_a / (t_comp / (2 * T)), "comm_comp_ratio_b": sync_b / (t_comp / (2 * T)),
        "hidden_fraction": 1.0 - (t_cross - t_comp) / sum_sync if sum_sync > 0 else None,
        "hidden_fraction_median_of_rounds": _median(per_round_hidden) if per_round_hidden else None,
        "hidden_fraction_per_round": per_round_hidden, "rounds": rounds,
        "speedup_vs_serial": t_serial / t_cross,
        "syncs_finished_before_compute_end": {"a": count[0] - late[0], "b": count[1] - late[1],
                                              "of_a": count[0], "of_b": count[1]},
        "hidden_b_no_stall": 1.0 - exposed[1] / (count[1] * sync_b) if count[1] else None,
        "hidden_a_no_stall": 1.0 - exposed[0] / (count[0] * sync_a) if count[0] else None,
    }
    for a in set(apps + apps_alone):
        a.destroy()
    return res


def cpu_baseline(w, align, budget_s=12.0):
    """The oracle as it stands on the same workload (bounded sample): one thread, as written,
    and with its element loop of the average + update spread over the host cores the process
    may use (pack and unpack stay single-threaded)."""
    import numpy as np
    import oracle
    from paper_2103_07974_amd import workloads as wl
    grads = [[t.numpy() for t in wl.make_replica_grads(w, r)] for r in range(w.W)]
    params0 = [t.numpy() for t in wl.make_params(w)]
    offs = oracle.layout(w.numel, align)
    lr, mu, wd = (np.float32(w.lr).item(), np.float32(w.momentum).item(),
                  np.float32(w.weight_decay).item())
    bytes_ = (w.W * w.grad_bytes + 16) * w.n_elems
    cores = len(os.sched_getaffinity(0))

    def run(threads, budget):
        params = params0
        v = np.zeros(int(offs[-1]))
        steps, t_total = 0, 0.0
        while steps < 2 or (t_total < budget and steps < 50):
            t0 = time.perf_counter()
            params, _ = oracle.sync_step(grads, params, v, lr, mu, wd, 1.0 / w.loss_scale,
                                         align=align, threads=threads)
            params = [p.astype(np.float32) for p in params]
            t_total += time.perf_counter() - t0
            steps += 1
        return steps, t_total * 1e3 / steps

    steps1, ms1 = run(1, budget_s)
    stepsn, msn = run(cores, budget_s / 2)
    return {"value": bytes_ / ms1 / 1e6, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "ms_per_step": ms1,
            "sample": f"{steps1} whole {w.name} steps (W={w.W} packs, double-precision "
                      f"reduce+SGD, unpack) of the C oracle, single thread, "
                      f"{cores} host cores available",
            "all_cores": {"value": bytes_ / msn / 1e6, "unit": "GB/s", "cores": cores,
                          "ms_per_step": msn,
                          "sample": f"{stepsn} of the same steps, the average + update loop under "
                                    f"OpenMP on {cores} threads, pack and unpack on one"}}


def traffic_probe():
    """A few launches for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: a plain device copy
    of known size first (its counter reading calibrates the unit), then the path's kernels
    on the headline workload."""
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
    for w in (wl.RESNET50, wl.VGG16):
        task = harness.make_task(w, "cuda")
        for _ in range(3):
            for r in range(w.W):
                xs.fuse_pack(task.gplan, task.grad_tables[r], task.buckets[r])
            xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum,
                                w.lr, w.momentum, w.weight_decay, 1.0)
            xs.fuse_unpack(task.pplan, task.params, task.param_table)
            xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, task.params,
                                       task.momentum, w.lr, w.momentum, w.weight_decay, 1.0,
                                       param_tensor_ptrs=task.param_table)
        torch.cuda.synchronize()
        print(json.dumps({"workload": w.name, "copy_bytes_each_way": n * 4,
                          "reduce_bytes": task.reduce_bytes(), "pack_bytes": task.pack_bytes(),
                          "unpack_bytes": task.unpack_bytes(), "gather_bytes": task.gather_bytes(True),
                          "bucket_elems": task.n_bucket}))
        del task
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--quick", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--crossover-only", action="store_true",
                    help="run only the crossover pair (T outer iterations), for rocprofv3 --kernel-trace")
    ap.add_argument("--T", type=int, default=20)
    ap.add_argument("--gather", action="store_true", help="with --crossover-only: gathering form")
    ap.add_argument("--autograd", action="store_true",
                    help="with --crossover-only: the two autograd MLP tasks instead of the GEMM-chain stand-in")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="launch a calibration copy and the path's kernels a few times (for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.traffic_probe:
        return traffic_probe()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the W workers' gradients are resident "
              "on that GPU); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2103_07974_amd import harness, workloads as wl, xs
    xs.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()

    if args.crossover_only and args.autograd:
        ma = harness.make_mlp_task("mlp_6x4096", [4096] * 7, W=4, batch=256, seed=31)
        mb = harness.make_mlp_task("mlp_8192_wide", [2048, 8192, 8192, 2048], W=4, batch=256, seed=32)
        print(json.dumps(crossover_pair(ma.state, mb.state, T=args.T, fused_gather=args.gather,
                                        cross_only=True, computes=(ma.compute, mb.compute),
                                        label="autograd forward+backward of two fp32 MLPs")))
        return 0
    if args.crossover_only:
        ta = harness.make_task(wl.RESNET50, "cuda")
        tb = harness.make_task(wl.VGG16, "cuda")
        print(json.dumps(crossover_pair(ta, tb, T=args.T, fused_gather=args.gather, cross_only=True)))
        return 0

    w = wl.RESNET50
    tasks = [harness.make_task(w, "cuda") for _ in range(3)]
    for t in tasks:   # steady state: momentum already non-zero
        t.momentum.copy_(wl.make_flat(t.n_bucket, 0.01, w.seed + 77, device="cuda"))
    ms_per_step, kernel_ms = time_steps(tasks, args.steps, args.warmup, stream)
    k_avg = sum(kernel_ms) / len(kernel_ms)
    reduce_bytes = tasks[0].reduce_bytes()
    achieved = reduce_bytes / k_avg / 1e6
    out = {
        "metric": "fused grad-sync GB/s + % HBM roofline; crossover sync-hidden fraction (1 GPU)",
        "value": reduce_bytes / ms_per_step / 1e6,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet50-shaped gradient set, 161 tensors, 25,557,032 elements, "
                               "W=8 fp32 replicas; step = 8 packs + fused reduce+SGD + unpack",
                   "W": w.W, "n_elems": w.n_elems, "n_tensors": w.n_tensors,
                   "bucket_align_elems": tasks[0].align,
                   "bytes_per_step_counted": reduce_bytes},
        "roofline": {"bound": "hbm", "kernel": "xs::reduce_sgd_kernel<8, 0, false, true, true, false>",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES,
                     "bytes_per_launch": reduce_bytes, "avg_launch_ms": k_avg,
                     "median_launch_ms": _median(kernel_ms), "min_launch_ms": min(kernel_ms)},
    }
    extra = {"resnet50": time_kernels(tasks[0], stream)}
    extra["resnet50"]["gather_form"] = time_gather(tasks, stream)
    extra["resnet50"]["param_groups"] = time_param_groups(tasks, stream)
    del tasks
    torch.cuda.empty_cache()

    if not args.quick:
        tiny = harness.make_task(wl.TINY_MLP, "cuda")
        tk = time_kernels(tiny, stream)
        app = tiny.make_app()
        with torch.cuda.stream(stream):
            for _ in range(20):
                app.sync(stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                app.sync(stream)
            torch.cuda.synchronize()
            tk["step_latency_us"] = (time.perf_counter() - t0) * 1e6 / 200
        app.destroy()
        # the same step as one gathering kernel, eager and replayed from a captured HIP graph
        app = tiny.make_app(fused_gather=True)
        with torch.cuda.stream(stream):
            for _ in range(20):
                app.sync(stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(200):
                app.sync(stream)
            torch.cuda.synchronize()
            tk["gather_step_latency_us"] = (time.perf_counter() - t0) * 1e6 / 200
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
        extra["tiny_mlp"] = {k: tk[k] for k in ("pack_ms", "reduce_sgd_ms", "unpack_ms", "step_latency_us",
                                                "gather_step_latency_us", "gather_step_latency_graph_us")}

        ta = harness.make_task(wl.RESNET50, "cuda")
        tb = harness.make_task(wl.VGG16, "cuda")
        extra["vgg16"] = time_kernels(tb, stream)
        with torch.cuda.stream(stream):
            app = tb.make_app()
            for _ in range(3):
                app.sync(stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                app.sync(stream)
            torch.cuda.synchronize()
            extra["vgg16"]["step_ms"] = (time.perf_counter() - t0) * 1e3 / 10
            app.destroy()
        extra["vgg16"]["gather_form"] = time_gather([tb], stream, reps=15, warm=3)
        extra["crossover"] = crossover_pair(ta, tb)
        extra["crossover_gather_form"] = crossover_pair(ta, tb, fused_gather=True)
        extra["crossover_alu_standin"] = crossover_pair(ta, tb, standin="alu")
        extra["crossover_alu_standin_gather_form"] = crossover_pair(ta, tb, fused_gather=True, standin="alu")
        del ta, tb
        torch.cuda.empty_cache()

        # a real forward + backward (autograd, fp32 MLPs of about 100 M parameters, one
        # micro-batch per worker) as each task's computation instead of a stand-in
        ma = harness.make_mlp_task("mlp_6x4096", [4096] * 7, W=4, batch=256, seed=31)
        mb = harness.make_mlp_task("mlp_8192_wide", [2048, 8192, 8192, 2048], W=4, batch=256, seed=32)
        lab = "autograd forward+backward of fp32 ReLU MLPs (6x4096^2 / 2048-8192-8192-2048), 4 micro-batches of 256"
        extra["crossover_autograd_mlp"] = crossover_pair(ma.state, mb.state, T=10, label=lab,
                                                         computes=(ma.compute, mb.compute))
        extra["crossover_autograd_mlp_gather_form"] = crossover_pair(
            ma.state, mb.state, T=10, label=lab, computes=(ma.compute, mb.compute), fused_gather=True)
        del ma, mb
        torch.cuda.empty_cache()

        bert = harness.make_task(wl.BERT_LARGE_F16, "cuda")
        extra["bert_large_f16"] = time_kernels(bert, stream, reps=15, warm=3)
        extra["bert_large_f16"]["gather_form"] = time_gather([bert], stream, reps=10, warm=2)
        extra["bert_large_f16"]["param_groups"] = time_param_groups([bert], stream, reps=10, warm=2)
        extra["bert_large_f16"]["overflow_skip"] = time_overflow_skip(bert, stream)
        del bert
        torch.cuda.empty_cache()

    if "crossover" in extra:
        c = extra["crossover"]
        out["crossover"] = {
            "config": "ResNet-50-shaped and VGG-16-shaped syncs beside " + c["compute_standin"] + f", T={c['T']}",
            "no_stall_fraction_app_b": c["hidden_b_no_stall"],
            "end_to_end_hidden_fraction": c["hidden_fraction"],
            "end_to_end_hidden_fraction_alu_standin": extra["crossover_alu_standin"]["hidden_fraction"],
            "stream_overlap_fraction_from_kernel_trace": STREAM_OVERLAP_FROM_TRACE,
            "speedup_vs_serial": c["speedup_vs_serial"],
        }
    out["extra"] = extra
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, harness.DEFAULT_ALIGN)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
