#!/usr/bin/env python3
"""Throughput of the batched schedule evaluation on one MI355X.

A step is one pass of the whole hot path (classification into geometric
batches, phase tables, start times, per-round occupancy, MemPeak, FlowTime)
over one batch of synthetic instances at every sweep point: one call of
kvs_gba_simulate.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` = simulated job-decode-steps per second;
`roofline` = algorithmic HBM bytes of the evaluation kernel over its measured
duration against the 8 TB/s peak; `cpu_baseline` = the CPU oracle timed on a
bounded sample of the same workload on this machine's host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
CHUNK = 4096                   # instances generated and uploaded at a time
HEAD = 4096                    # instances at the front of the workload the oracle may be run on
TRAFFIC_NOTE = os.path.join(ROOT, "profiles", "kvs_sweep_kernel_cfg5_pareto_traffic.md")


def kernel_source_digest():
    """sha256 over the code of the sources the evaluation kernel is built from (comments and
    white space do not count: they do not change the kernel)."""
    import hashlib
    import re
    h = hashlib.sha256()
    for rel in ("paper_2601_22996_amd/csrc/kvs_kernels.hip", "paper_2601_22996_amd/csrc/kvs_phase.h",
                "paper_2601_22996_amd/csrc/kvs_wave.h", "paper_2601_22996_amd/csrc/kvs_math.h"):
        with open(os.path.join(ROOT, rel), "r") as f:
            code = re.sub(r"/\*.*?\*/|//[^\n]*", " ", f.read(), flags=re.S)
        h.update(" ".join(code.split()).encode())
    return h.hexdigest()


def measured_counters(workload_name):
    """The key: value lines of the committed rocprofv3 --pmc note, or {} when the note is for
    another workload or the kernel sources have changed since the counters were taken."""
    try:
        text = open(TRAFFIC_NOTE).read()
    except OSError:
        return {}
    kv = dict(line.strip("- ").split(": ", 1) for line in text.splitlines()
              if line.startswith("- ") and ": " in line)
    if kv.get("workload") != workload_name or kv.get("source_sha256") != kernel_source_digest():
        return {}
    return kv


def measured_traffic(workload_name):
    """HBM bytes per launch (scaled FETCH_SIZE + WRITE_SIZE), or None."""
    kv = measured_counters(workload_name)
    return int(kv["traffic_bytes_per_launch"]) if "traffic_bytes_per_launch" in kv else None


def load_workload(w, torch, threads):
    """Generate the whole workload on the host, chunk by chunk, into device tensors."""
    from paper_2601_22996_amd import workloads as W
    I, n = w.n_instances, w.n_jobs
    dev = torch.device("cuda:0")
    o = torch.empty((I, n), dtype=torch.int32, device=dev)
    s = torch.empty((I, n), dtype=torch.int32, device=dev) if w.s_scalar is None else None
    e = torch.empty((I, n), dtype=torch.int32, device=dev) if w.estimates else None
    buf = None
    for i0 in range(0, I, CHUNK):
        i1 = min(I, i0 + CHUNK)
        buf = W.generate(w, i0, i1, threads=threads, out=buf)
        o[i0:i1].copy_(torch.from_numpy(buf["o"]))
        if s is not None:
            s[i0:i1].copy_(torch.from_numpy(buf["s"]))
        if e is not None:
            e[i0:i1].copy_(torch.from_numpy(buf["o_est"]))
    torch.cuda.synchronize()
    return o, s, e


def cpu_baseline(w, pts, target_seconds, threads, gpu_head):
    """The oracle as it stands on the first instances of the workload: first on one core, then
    one oracle call per thread over disjoint instance ranges (instances are independent; the
    oracle itself is single-threaded and the C call releases the interpreter lock).  Outside
    the timing, everything the oracle computed is compared with the GPU's results for the
    same instances (`gpu_head`: the outputs of the first instances, on the host)."""
    import numpy as np
    import oracle as O
    from concurrent.futures import ThreadPoolExecutor
    from paper_2601_22996_amd import workloads as W
    probe = min(4, w.n_instances)
    d = W.generate(w, 0, min(w.n_instances, HEAD))
    avail = d["o"].shape[0]
    sarg = d["s"] if d["s"] is not None else d["s_scalar"]
    kept = []

    def run(i0, i1):
        if w.mode == W.MODE_GBAD:
            r = O.gbad_simulate_batch(d["o"], sarg, d["M"], [tuple(p[:3]) for p in pts], i0, i1)
        else:
            r = O.gba_simulate_batch(d["o"], sarg, d["M"], pts, d["o_est"], i0, i1)
        kept.append((i0, i1, r))
        return int(r["job_steps"].sum())

    t = time.perf_counter()
    run(0, probe)
    per_inst = max(time.perf_counter() - t, 1e-6) / probe
    half = target_seconds / 2
    cnt1 = int(max(probe, min(avail, half / per_inst)))
    t = time.perf_counter()
    steps1 = run(0, cnt1)
    dt1 = time.perf_counter() - t
    threads = max(1, min(threads, avail))
    per = int(max(1, min(avail // threads, half / per_inst)))
    cuts = [(j * per, (j + 1) * per) for j in range(threads)]
    with ThreadPoolExecutor(threads) as ex:
        t = time.perf_counter()
        stepsN = sum(ex.map(lambda c: run(*c), cuts))
        dtN = time.perf_counter() - t
    checked = np.zeros(avail, bool)
    mismatches = 0
    for i0, i1, r in kept:
        for key in ("peak", "feasible", "flow", "job_steps"):
            mismatches += int((r[key] != gpu_head[key][:, i0:i1]).sum())
        checked[i0:i1] = True
    return {"value": stepsN / dtN, "unit": "job-decode-steps/s", "cores": threads, "kind": "oracle",
            "value_1core": steps1 / dt1,
            "checked_evaluations": int(checked.sum()) * len(pts), "mismatches": mismatches,
            "sample": f"literal round-by-round stepping in C (-O2) at all {len(pts)} sweep points: instances "
                      f"0..{threads * per - 1} of the workload in {threads} disjoint ranges on {threads} threads, "
                      f"{stepsN} job-steps in {dtN:.1f} s; one core alone: instances 0..{cnt1 - 1}, "
                      f"{steps1} job-steps in {dt1:.1f} s"}


def timed(torch, steps, warmup, call):
    """ms per step by wall clock around `steps` calls, and by events on the calls' stream."""
    for _ in range(warmup):
        call()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        call()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall * 1e3 / steps, sum(a.elapsed_time(b) for a, b in ev) / steps


def bench_bounds(args, torch, K, W):
    """The evaluators that frame the flow time: kvs_flow_bounds on the workload's instances at the
    initial slices 1..128, or kvs_opt_perm on 4096 instances of the 8-job workload's shape."""
    import oracle as O
    import numpy as np
    if args.path == "bounds":
        w = W.WORKLOADS[args.config]
        tau0 = [1, 2, 4, 8, 16, 32, 64, 128]
        o, s, _ = load_workload(w, torch, args.threads)
        sarg = s if s is not None else w.s_scalar
        out = K.flow_bounds(o, sarg, w.M, tau0)
        ms_step, kern_ms = timed(torch, args.steps, args.warmup,
                                 lambda: K.flow_bounds(o, sarg, w.M, tau0, out=out))
        assert int(out["upper_gba"].min().item()) > 0 and int(out["area_lb_num"].min().item()) > 0
        n_eval = w.n_instances * (len(tau0) + 1)
        alg_bytes = w.n_instances * (w.n_jobs * 4 * (1 + (s is not None)) + 8 * (len(tau0) + 1))
        res = {"metric": "bounds (UpperGBA per initial slice + area lower bound) per second on 1 MI355X",
               "value": n_eval / (ms_step * 1e-3), "unit": "bounds/s",
               "config": {"workload": w.name, "n_instances": w.n_instances, "n_jobs": w.n_jobs, "M": w.M,
                          "initial_slices": len(tau0)},
               "kernel": "kvs_bounds_kernel"}
        cpu = None
        if args.cpu_seconds > 0:
            d = W.generate(w, 0, 64)
            sh = d["s"] if d["s"] is not None else None
            t0, cnt = time.perf_counter(), 0
            while time.perf_counter() - t0 < args.cpu_seconds / 2 and cnt < 64:
                si = sh[cnt] if sh is not None else d["s_scalar"]
                for t in tau0:
                    O.upper_gba(d["o"][cnt], si, w.M, t)
                O.area_lb(d["o"][cnt], si)
                cnt += 1
            dt = time.perf_counter() - t0
            cpu = {"value": cnt * (len(tau0) + 1) / dt, "unit": "bounds/s", "cores": 1, "kind": "oracle",
                   "sample": f"instances 0..{cnt - 1} of the workload, {len(tau0)} slices + area bound each, {dt:.1f} s"}
    else:
        w = W.WORKLOADS[1]
        I = 4096
        rng = np.random.default_rng(0)
        oh = rng.integers(1, 33, (I, w.n_jobs)).astype(np.int32)       # config 1's shape: 8 jobs, o in 1..32
        o = torch.from_numpy(oh).cuda()
        out = K.opt_perm(o, w.s_scalar, w.M)
        ms_step, kern_ms = timed(torch, args.steps, args.warmup,
                                 lambda: K.opt_perm(o, w.s_scalar, w.M, out=out))
        orders = 40320 * I
        alg_bytes = I * (w.n_jobs * 4 + 8)
        res = {"metric": "list schedules (orders of an 8-job instance) evaluated per second on 1 MI355X",
               "value": orders / (ms_step * 1e-3), "unit": "orders/s",
               "config": {"workload": "cfg1_shape_x4096", "n_instances": I, "n_jobs": w.n_jobs, "M": w.M,
                          "s": w.s_scalar, "orders_per_instance": 40320},
               "kernel": "kvs_opt_perm_kernel"}
        cpu = None
        if args.cpu_seconds > 0:
            t0, cnt = time.perf_counter(), 0
            while time.perf_counter() - t0 < args.cpu_seconds / 2 and cnt < I:
                assert O.opt_perm(oh[cnt], w.s_scalar, w.M) == int(out[cnt].item())
                cnt += 1
            dt = time.perf_counter() - t0
            cpu = {"value": cnt * 40320 / dt, "unit": "orders/s", "cores": 1, "kind": "oracle",
                   "sample": f"instances 0..{cnt - 1} (all orders each, results equal to the GPU's), {dt:.1f} s"}
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    res.update({"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
                "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64",
                "data": "synthetic",
                # inputs read once + outputs against the memory peak; neither kernel is limited by memory:
                # the ranking of the areas lives in LDS and registers, the list schedules are integer ALU work
                "roofline": {"bound": "alu", "bound_detail": "valu-issue (integer vector instructions)",
                             "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": res.pop("kernel"),
                             "kernel_ms": kern_ms, "algorithmic_bytes_per_launch": alg_bytes}})
    if cpu:
        res["cpu_baseline"] = cpu
    print(json.dumps(res))


def copy_bandwidth(torch):
    """Read + write rate of a plain 1 GiB device-to-device copy, GB/s: what this GPU's memory
    delivers to the simplest kernel there is, for scale next to the nominal peak."""
    src = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0").random_(0, 1000)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 5 * 2 * src.numel() * 4 / (a.elapsed_time(b) * 1e-3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the largest sweep)")
    ap.add_argument("--instances", type=int, default=0, help="override the workload's number of instances")
    ap.add_argument("--jobs", type=int, default=0, help="override the workload's jobs per instance")
    ap.add_argument("--mode", choices=["workload", "gsa", "gbad"], default="workload",
                    help="gsa: the workload's sweep in GSA mode (Algorithm 1: every unfinished job in every phase); "
                         "gbad: with dynamic refill (GBA-D)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="wall time of the oracle baseline (half on one core, half on all threads); 0 skips it")
    ap.add_argument("--threads", type=int, default=min(16, os.cpu_count() or 1))
    ap.add_argument("--path", choices=["sweep", "bounds", "opt_perm"], default="sweep",
                    help="sweep: the schedule evaluation (default); bounds: UpperGBA and the area lower "
                         "bound on the same workload; opt_perm: best order of 8-job instances by brute force")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies: a kernel of known traffic "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on ONE GPU (instances are independent; more GPUs would "
                 "each take a slice of the instance axis). Run with --gpus 1.")

    import dataclasses
    import statistics
    import torch
    from paper_2601_22996_amd import kvsched as K
    from paper_2601_22996_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    K.lib()
    if args.path != "sweep":
        return bench_bounds(args, torch, K, W)
    w = W.WORKLOADS[args.config]
    if args.instances or args.jobs:
        w = dataclasses.replace(w, n_instances=args.instances or w.n_instances, n_jobs=args.jobs or w.n_jobs)
        w = dataclasses.replace(w, name=f"{w.name}_{w.n_instances}x{w.n_jobs}")
    if args.mode == "gsa":
        w = dataclasses.replace(w, mode=W.MODE_GSA, name=w.name + "_gsa")
    if args.mode == "gbad":
        w = dataclasses.replace(w, mode=W.MODE_GBAD, estimates=False, name=w.name + "_gbad")
    pts = w.sweep()
    o, s, e = load_workload(w, torch, args.threads)
    sarg = s if s is not None else w.s_scalar
    out = K.gba_simulate(o, sarg, w.M, pts, o_est=e)          # allocates the outputs once
    torch.cuda.synchronize()

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0").random_(0, 1000)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        K.gba_simulate(o, sarg, w.M, pts, o_est=e, out=out)
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()                                            # same stream as the kernel
        K.gba_simulate(o, sarg, w.M, pts, o_est=e, out=out)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    kern_ms = statistics.median(a.elapsed_time(b) for a, b in ev)
    job_steps = int(out["job_steps"].sum().item())
    feas = out["feasible"]
    assert int(feas.max().item()) <= 1, "an evaluation reported an in-band error"
    copy_gbs = copy_bandwidth(torch)

    bytes_per_job = 4 * (1 + (s is not None) + (e is not None))
    n_eval = w.n_instances * len(pts)
    alg_bytes = n_eval * (w.n_jobs * bytes_per_job + 25)
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    fused_bytes = w.n_instances * w.n_jobs * bytes_per_job + n_eval * 25
    kv = measured_counters(w.name)
    valu = int(kv["valu_wave_instructions_per_launch"]) if "valu_wave_instructions_per_launch" in kv else None
    traffic = measured_traffic(w.name)
    res = {
        "metric": "simulated job-decode-steps/sec on 1 MI355X + % of HBM roofline",
        "value": job_steps / (ms_step * 1e-3),
        "unit": "job-decode-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name, "n_instances": w.n_instances, "n_jobs": w.n_jobs,
                   "M": w.M, "sweep_points": len(pts), "job_steps_per_step": job_steps,
                   "evaluations_per_step": n_eval},
        # `achieved`, `peak`, `frac`: the metric's own accounting -- the bytes an evaluation must read and
        # write (each sweep point counted as if it read its instance), a statement about evaluations per
        # second.  It is NOT the utilisation of the memory bus: the kernel reads an instance once for all
        # its sweep points (`hbm_physical_frac`), and what it runs into is the issue rate of integer
        # vector instructions (`bound`, `valu_issue_frac`).
        "roofline": {"bound": "alu",
                     "bound_detail": ("latency of dependent LDS operations: one wavefront per evaluation, sequential by nature"
                                      if w.mode == W.MODE_GBAD else
                                      "valu-issue (integer vector instructions), then the LDS pipeline"),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "kvs_gbad_kernel" if w.mode == W.MODE_GBAD else "kvs_sweep_kernel",
                     "kernel_ms": kern_ms, "kernel_ms_is": "median of the steps",
                     "algorithmic_bytes_per_launch": alg_bytes,
                     # the fused kernel reads an instance once per launch, not once per point
                     "fused_bytes_per_launch": fused_bytes,
                     "achieved_fused": fused_bytes / (kern_ms * 1e-3) / 1e9,
                     "hbm_physical_frac": (traffic if traffic is not None else fused_bytes) / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "hbm_physical_from": "rocprofv3 FETCH_SIZE + WRITE_SIZE" if traffic is not None else "inputs once + outputs",
                     "copy_bandwidth_GBs": copy_gbs,
                     # issue slots: a vector instruction holds one of 1024 SIMDs for 4 cycles at 2.4 GHz;
                     # the instruction count is rocprofv3's SQ_INSTS_VALU of the same kernel (null when the
                     # sources have changed since it was taken)
                     "valu_issue_frac": None if valu is None else valu * 4 / (1024 * 2.4e9 * kern_ms * 1e-3)},
    }
    rc = 0
    if args.cpu_seconds > 0:
        head = min(HEAD, w.n_instances)
        gpu_head = {k: out[k][:, :head].cpu().numpy() for k in ("peak", "feasible", "flow", "job_steps")}
        res["cpu_baseline"] = cpu_baseline(w, pts, args.cpu_seconds, args.threads, gpu_head)
        rc = 2 if res["cpu_baseline"]["mismatches"] else 0
    print(json.dumps(res))
    if rc:
        sys.exit("bench.py: the GPU results differ from the oracle's on the instances the baseline ran")


if __name__ == "__main__":
    main()
