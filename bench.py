#!/usr/bin/env python3
"""Benchmark of the CAME optimizer step on one MI355X.

A "step" is one full came_step (sweep 1, finalize 1, sweep 2, finalize 2,
sweep 3 over every tensor) on a synthetic Llama-6.7B-shaped parameter list
with bf16 gradients and fp32 parameters/state, all resident in HBM before the
timed region.  Prints ONE JSON line:

  value        parameters updated per second (whole step, wall clock around K steps)
  roofline     the dominant kernel (sweep 3: reads g, M, theta, writes M, theta) --
               algorithmic bytes per launch / mean launch time, the latter taken
               with HIP events on the step's stream inside the timed region
               (came_profile_enable / came_profile_read)
  cpu_baseline the double-precision CPU oracle timed on the host cores on a
               bounded sample of the same workload (a baseline, not the target)
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def read_traffic(path: str):
    """HBM bytes per sweep-3 launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    as recorded in a text summary under profiles/; None when no summary is there."""
    if not os.path.exists(path):
        return None
    vals = dict(re.findall(r"^(\w+)\s*:\s*([0-9.eE+-]+)\s*$", open(path).read(), flags=re.M))
    try:
        return float(vals["fetch_bytes_per_launch"]) + float(vals["write_bytes_per_launch"])
    except KeyError:
        return None


def cpu_baseline(w, gen, hyper, lr, budget_s: float = 12.0):
    """Times oracle steps on layers 0 and 1 of the list (every distinct per-layer shape),
    one tensor per OpenMP thread, until about budget_s seconds have been spent."""
    import numpy as np
    from oracle import came_oracle as O

    first = next(i for i, s in enumerate(w.shapes) if len(s) == 2) + 1  # skip the embedding
    per_layer = 9
    idx = list(range(min(first, len(w.shapes) - 1), min(first + 2 * per_layer, len(w.shapes))))
    shapes = [w.shapes[i] for i in idx]
    n_params = sum(math.prod(s) for s in shapes)
    to64 = lambda t: t.detach().to("cpu").float().numpy().astype(np.float64)
    tl = O.TensorList(shapes, [to64(gen.theta0(i)) for i in idx])
    grads = [to64(gen.grad(i, 1)) for i in idx]
    oh = O.Hyper(hyper.beta1, hyper.beta2, hyper.beta3, hyper.eps1, hyper.eps2, hyper.clip_d, lr)
    threads = min(O.max_threads(), len(idx))
    steps, t0 = 0, time.perf_counter()
    while True:
        tl.step(grads, oh, nthreads=threads)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or steps >= 50:
            break
    # the same oracle on one thread: one step of one attention projection
    one = next(k for k, s in enumerate(shapes) if len(s) == 2)
    tl1 = O.TensorList([shapes[one]], [to64(gen.theta0(idx[one]))])
    t2 = time.perf_counter()
    tl1.step([grads[one]], oh, nthreads=1)
    dt1 = time.perf_counter() - t2
    return {
        "value": n_params * steps / dt,
        "unit": "params/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"{steps} step(s) of tensors {idx[0]}..{idx[-1]} (two transformer layers, "
                  f"{len(idx)} tensors, {n_params} params), one tensor per thread, float64",
        "seconds": dt,
        "single_thread": {"value": math.prod(shapes[one]) / dt1, "unit": "params/s", "cores": 1,
                          "sample": f"1 step of tensor {idx[one]} {tuple(shapes[one])}", "seconds": dt1},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama_7b")
    ap.add_argument("--tile-rows", type=int, default=0)
    ap.add_argument("--group-elements", type=int, default=0)
    ap.add_argument("--momentum-dtype", choices=("f32", "bf16"), default="f32",
                    help="storage type of the momentum M between steps (f32: the configuration the metric is "
                         "quoted on; bf16: the reduced-precision-momentum variant, 6 bytes per parameter less)")
    ap.add_argument("--grad-dtype", choices=("workload", "f32", "bf16"), default="workload",
                    help="gradient storage type: the workload's own (default), or overridden to see the other "
                         "kernel variants at the same shapes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=12.0)
    ap.add_argument("--no-placement", action="store_true",
                    help="allocate the state blob wherever the allocator puts it (default: probe several "
                         "addresses against the parameters and keep the fastest)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 4 GiB device-to-device copy a few times: the known-size kernel "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    import paper_2307_02047_amd as P
    from paper_2307_02047_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    if args.calibrate_copy:
        n = (4 << 30) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n * 4, "calibrate_copy_bytes_written": n * 4,
                          "launches": 4}), flush=True)
        return 0
    w = W.by_name(args.workload)
    if args.grad_dtype != "workload":
        import dataclasses
        w = dataclasses.replace(w, grad_dtype=W.GRAD_F32 if args.grad_dtype == "f32" else W.GRAD_BF16)
    gen = W.Generator(w, device=dev)
    n = len(w.shapes)
    hyper = P.CameHyper()
    lr = w.lr

    theta = [gen.theta0(i) for i in range(n)]
    # two gradient sets, alternated step by step, so that no random numbers are drawn inside the timed region
    grad_sets = [[gen.grad(i, t) for i in range(n)] for t in (1, 2)]
    mdt = P.MOMENTUM_BF16 if args.momentum_dtype == "bf16" else P.MOMENTUM_F32
    mbytes = 2 if mdt == P.MOMENTUM_BF16 else 4
    opt = P.CameStep(w.shapes, [w.grad_dtype] * n, device=dev, tile_rows=args.tile_rows,
                     group_elements=args.group_elements, momentum_dtype=mdt,
                     place_against=None if args.no_placement else theta)
    opt.check_tensors(theta, grad_sets[0])
    plan = P.plan_query(w.shapes, [w.grad_dtype] * n, tile_rows=args.tile_rows,
                        group_elements=args.group_elements)
    torch.cuda.synchronize()

    step_no = 0
    for _ in range(args.warmup):
        step_no += 1
        opt.step(theta, grad_sets[step_no % 2], hyper, lr, step_no)
    torch.cuda.synchronize()

    # one event before each step and one after the last, on the stream the steps run on:
    # per-step durations (median, min) beside the wall-clock mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    opt.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step_no += 1
        marks[k].record()
        opt.step(theta, grad_sets[step_no % 2], hyper, lr, step_no)
    marks[args.steps].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    opt.profile_enable(False)
    phases = opt.profile_read()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    step_ms = {"median": per_step[len(per_step) // 2] if len(per_step) % 2 else
               0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2]),
               "min": per_step[0], "max": per_step[-1]}
    n_params = w.n_params
    n_matrix_params = sum(s[0] * s[1] for s in w.shapes if len(s) == 2)
    value = n_params / (ms_per_step * 1e-3)

    gb = w.grad_bytes
    s3_ms, s3_launches = phases["sweep3"]
    s3_avg_ms = s3_ms / max(s3_launches, 1)
    # one sweep-3 launch covers every matrix element of a launch group
    units_per_launch = n_matrix_params * (args.steps / max(s3_launches, 1))
    step_bpp = P.algorithmic_bytes(gb, mbytes, P.ALGO_CAME, 0)
    s3_bytes = P.algorithmic_bytes(gb, mbytes, P.ALGO_CAME, 3) * units_per_launch
    achieved = s3_bytes / (s3_avg_ms * 1e-3) / 1e9 if s3_avg_ms > 0 else 0.0
    roofline = {
        "bound": "hbm",
        "kernel": "sweep3_kernel",
        "achieved": achieved,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS,
        "traffic": read_traffic(os.path.join(
            ROOT, "profiles", f"sweep3_{args.workload}{'_bf16_momentum' if mbytes == 2 else ''}_traffic.txt"))
        if args.grad_dtype == "workload" else None,
        "bytes_per_launch": s3_bytes,
        "avg_launch_ms": s3_avg_ms,
        "whole_step": {
            "algorithmic_bytes_per_param": step_bpp,
            "achieved_GBs": step_bpp * n_params / (ms_per_step * 1e-3) / 1e9,
            "frac": step_bpp * n_params / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        },
        "phase_ms_per_step": {k: v[0] / args.steps for k, v in phases.items()},
    }

    out = {
        "metric": "CAME step params updated/sec and achieved HBM GB/s (% of peak), 1 MI355X",
        "value": value,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "step_ms": step_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name,
            "params": n_params,
            "tensors": n,
            "grad_dtype": "bf16" if gb == 2 else "f32",
            "param_state_dtype": "f32",
            "momentum_dtype": args.momentum_dtype,
            "tile_rows": plan["tile_rows"],
            "launch_groups": plan["groups"],
            "state_placement_probe_GBs": [round(g, 1) for _, g in opt.placement_log],
        },
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, gen, hyper, lr, args.cpu_budget)
    opt.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
