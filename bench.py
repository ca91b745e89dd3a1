#!/usr/bin/env python3
"""Benchmark of the CAME optimizer step on one MI355X.

A "step" is one full came_step (sweep 1, finalize 1, sweep 2, finalize 2,
sweep 3 over every tensor) on a synthetic Llama-6.7B-shaped parameter list
with bf16 gradients and fp32 parameters/state, all resident in HBM before the
timed region.  Prints ONE JSON line:

  value        parameters updated per second (whole step, wall clock around K steps), with the
               state blob placed by came_probe_placement
  no_placement the same steps with the state blob where the allocator put it by itself
  other_workloads  the BERT-Base-, GPT-2-medium- and BERT-Large-shaped lists, timed in the same
               process after the headline: placed, unplaced, and ("on_chip") with the matrices
               that fit on the on-chip path of came_options.resident, which moves a third fewer
               bytes and is off by default because it measures slower
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


def ceilings(torch, dev) -> int:
    """What this card's memory system gives to plain streaming kernels that are not ours
    (PyTorch's elementwise / reduction kernels on 4 GiB buffers): the yardstick beside the 8 TB/s
    the roofline is priced against."""
    n = (4 << 30) // 4
    x = torch.ones(n, dtype=torch.float32, device=dev)
    y = torch.ones(n, dtype=torch.float32, device=dev)
    z = torch.empty(n, dtype=torch.float32, device=dev)
    cases = {
        "read_only_sum": (lambda: torch.sum(x), 4 * n),
        "write_only_fill": (lambda: z.fill_(1.0), 4 * n),
        "read_write_in_place_mul": (lambda: x.mul_(1.0), 8 * n),
        "copy": (lambda: z.copy_(x), 8 * n),
        "two_reads_one_write_add": (lambda: torch.add(x, y, out=z), 12 * n),
    }
    out = {}
    for name, (fn, nbytes) in cases.items():
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name] = {"GBs": nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9, "bytes_per_launch": nbytes}
    print(json.dumps({"ceilings": out, "buffer_bytes": 4 * n, "peak_GBs": HBM_PEAK_GBS}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama_7b")
    ap.add_argument("--tile-rows", type=int, default=0, help="rows per tile of sweeps 1 and 2 (0: chosen from the list)")
    ap.add_argument("--tile-rows3", type=int, default=0, help="rows per tile of the update sweep (0: the library's default: 16, or 32 with the bfloat16 momentum)")
    ap.add_argument("--group-elements", type=int, default=0)
    ap.add_argument("--momentum-dtype", choices=("f32", "bf16"), default="f32",
                    help="storage type of the momentum M between steps (f32: the configuration the metric is "
                         "quoted on; bf16: the reduced-precision-momentum variant, 6 bytes per parameter less)")
    ap.add_argument("--grad-dtype", choices=("workload", "f32", "bf16"), default="workload",
                    help="gradient storage type: the workload's own (default), or overridden to see the other "
                         "kernel variants at the same shapes")
    ap.add_argument("--resident", choices=("auto", "off", "on"), default="auto",
                    help="the on-chip path for matrices whose tiles all fit on the chip (came_options.resident); "
                         "auto = the library's default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=12.0)
    ap.add_argument("--no-placement", action="store_true",
                    help="allocate the state blob wherever the allocator puts it (default: probe several "
                         "addresses against the parameters and keep the fastest)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the BERT-Base-, GPT-2-medium- and BERT-Large-shaped lists that the default run times "
                         "after the headline workload")
    ap.add_argument("--other-steps", type=int, default=200)
    ap.add_argument("--ceilings", action="store_true",
                    help="only time PyTorch's own streaming kernels (sum, fill, in-place multiply, copy, add) on "
                         "4 GiB buffers: what the memory system gives to kernels that are not this library's")
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
    if args.ceilings:
        return ceilings(torch, dev)
    w = W.by_name(args.workload)
    if args.grad_dtype != "workload":
        import dataclasses
        w = dataclasses.replace(w, grad_dtype=W.GRAD_F32 if args.grad_dtype == "f32" else W.GRAD_BF16)
    hyper = P.CameHyper()
    mdt = P.MOMENTUM_BF16 if args.momentum_dtype == "bf16" else P.MOMENTUM_F32
    mbytes = 2 if mdt == P.MOMENTUM_BF16 else 4
    resident = {"auto": P.RESIDENT_AUTO, "off": P.RESIDENT_OFF, "on": P.RESIDENT_ON}[args.resident]

    def run(w, steps, warmup, placement, resident=resident):
        """Times `steps` came_step calls on workload w (after `warmup` untimed ones), everything
        resident in HBM beforehand.  Returns (figures, context, generator); the caller closes the context."""
        gen = W.Generator(w, device=dev)
        n = len(w.shapes)
        theta = [gen.theta0(i) for i in range(n)]
        # two gradient sets, alternated step by step: no random numbers are drawn inside the timed region
        grad_sets = [[gen.grad(i, t) for i in range(n)] for t in (1, 2)]
        opt = P.CameStep(w.shapes, [w.grad_dtype] * n, device=dev, tile_rows=args.tile_rows, tile_rows3=args.tile_rows3,
                         group_elements=args.group_elements, momentum_dtype=mdt, resident=resident,
                         place_against=theta if placement else None,
                         place_against_grads=grad_sets[0] if placement else None)
        opt.check_tensors(theta, grad_sets[0])
        torch.cuda.synchronize()
        step_no = 0
        for _ in range(warmup):
            step_no += 1
            opt.step(theta, grad_sets[step_no % 2], hyper, w.lr, step_no)
        torch.cuda.synchronize()
        # one event before each step and one after the last, on the stream the steps run on:
        # per-step durations (median, min) beside the wall-clock mean
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        opt.profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            step_no += 1
            marks[k].record()
            opt.step(theta, grad_sets[step_no % 2], hyper, w.lr, step_no)
        marks[steps].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        opt.profile_enable(False)
        phases = opt.profile_read()
        ms = (t1 - t0) * 1e3 / steps
        per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
        mid = len(per_step) // 2
        gb = w.grad_bytes
        n_matrix = sum(s[0] * s[1] for s in w.shapes if len(s) == 2)
        # what the plan moves: streamed matrices 8 + 3 g + 3 M bytes per element, matrices on the
        # on-chip path 8 + g + 2 M, 1-D parameters 24 + g + 2 M
        traffic = P.plan_traffic(w.shapes, [w.grad_dtype] * n, tile_rows=args.tile_rows, group_elements=args.group_elements,
                                 momentum_dtype=mdt, resident=resident)
        bpp = traffic["bytes_per_step"] / w.n_params
        bpp_stream = traffic["bytes_per_step_streaming"] / w.n_params
        bmin = 8.0 + gb + 2.0 * mbytes  # every array crosses once: g, M read, M written, theta read and written
        s3_ms, s3_launches = phases["sweep3"]
        s3_avg = s3_ms / max(s3_launches, 1)
        s3_bytes = (P.algorithmic_bytes(gb, mbytes, P.ALGO_CAME, 3) * (n_matrix - traffic["resident_elements"]) *
                    (steps / max(s3_launches, 1)))
        fig = {
            "ms_per_step": ms,
            "step_ms": {"median": per_step[mid] if len(per_step) % 2 else 0.5 * (per_step[mid - 1] + per_step[mid]),
                        "min": per_step[0], "max": per_step[-1]},
            "value": w.n_params / (ms * 1e-3),
            "bytes_per_param": bpp,
            "whole_step_GBs": bpp * w.n_params / (ms * 1e-3) / 1e9,
            "whole_step_frac": bpp * w.n_params / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            # the same time priced as if every matrix had taken the three streaming sweeps
            # (20 + 3 sizeof(g) bytes per parameter): comparable across plans, not a bandwidth
            "streaming_bytes_per_param": bpp_stream,
            "streaming_equivalent_frac": bpp_stream * w.n_params / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "on_chip_matrices": traffic["resident_matrices"],
            "on_chip_elements": traffic["resident_elements"],
            "bmin_bytes_per_param": bmin,
            "bmin_frac": bmin * w.n_params / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "sweep3_avg_launch_ms": s3_avg,
            "sweep3_bytes_per_launch": s3_bytes,
            "sweep3_GBs": s3_bytes / (s3_avg * 1e-3) / 1e9 if s3_avg > 0 else 0.0,
            "phase_ms_per_step": {k: v[0] / steps for k, v in phases.items()},
            "placement_probe_GBs": [round(g, 1) for _, g in opt.placement_log],
        }
        del grad_sets
        return fig, opt, gen

    n = len(w.shapes)
    plan = P.plan_query(w.shapes, [w.grad_dtype] * n, tile_rows=args.tile_rows, group_elements=args.group_elements,
                        resident=resident)
    gb = w.grad_bytes

    # The state blob where the allocator puts it by itself (what a caller gets who does not use
    # came_probe_placement), then -- unless switched off -- the placed one, which is the headline.
    plain, plain_opt, gen = run(w, args.steps, args.warmup, placement=False)
    if args.no_placement:
        fig, opt = plain, plain_opt
    else:
        fig, opt, gen = run(w, args.steps, args.warmup, placement=True)  # the plain blob stays allocated meanwhile
        plain_opt.close()
    del plain_opt

    ms_per_step = fig["ms_per_step"]
    roofline = {
        "bound": "hbm",
        "kernel": "sweep3_kernel",
        "achieved": fig["sweep3_GBs"],
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": fig["sweep3_GBs"] / HBM_PEAK_GBS,
        "traffic": read_traffic(os.path.join(
            ROOT, "profiles", f"sweep3_{args.workload}{'_bf16_momentum' if mbytes == 2 else ''}_traffic.txt"))
        if args.grad_dtype == "workload" else None,
        "traffic_source": "replayed from the committed rocprofv3 --pmc summary under profiles/ (FETCH_SIZE and "
                          "WRITE_SIZE need runs of their own); not measured in this run",
        "bytes_per_launch": fig["sweep3_bytes_per_launch"],
        "avg_launch_ms": fig["sweep3_avg_launch_ms"],
        "whole_step": {
            "streaming_bytes_per_param": fig["streaming_bytes_per_param"],
            "streaming_equivalent_frac": fig["streaming_equivalent_frac"],
            "on_chip_matrices": fig["on_chip_matrices"],
            "on_chip_elements": fig["on_chip_elements"],
            "algorithmic_bytes_per_param": fig["bytes_per_param"],
            "achieved_GBs": fig["whole_step_GBs"],
            "frac": fig["whole_step_frac"],
            # the conservative figure: priced as if every array crossed the memory bus only once
            "bmin_bytes_per_param": fig["bmin_bytes_per_param"],
            "bmin_frac": fig["bmin_frac"],
        },
        "phase_ms_per_step": fig["phase_ms_per_step"],
    }

    out = {
        "metric": "CAME step params updated/sec and achieved HBM GB/s (% of peak), 1 MI355X",
        "value": fig["value"],
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "step_ms": fig["step_ms"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name,
            "params": w.n_params,
            "tensors": n,
            "grad_dtype": "bf16" if gb == 2 else "f32",
            "param_state_dtype": "f32",
            "momentum_dtype": args.momentum_dtype,
            "tile_rows": plan["tile_rows"],
            "tile_rows_update_sweep": args.tile_rows3 or (16 if args.momentum_dtype == "bf16" else 12),
            "launch_groups": plan["groups"],
            "state_placement_probe_GBs": fig["placement_probe_GBs"],
        },
        "roofline": roofline,
        # the same list, same steps, with the state blob where the allocator put it (no search)
        "no_placement": {k: plain[k] for k in ("ms_per_step", "value", "whole_step_frac", "bmin_frac", "sweep3_GBs",
                                               "streaming_equivalent_frac",
                                               "phase_ms_per_step")},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, gen, hyper, w.lr, args.cpu_budget)
    opt.close()
    del opt, gen
    torch.cuda.empty_cache()

    # The lists shaped like the paper's own models (BERT-Base, GPT-2 medium, BERT-Large), timed in
    # the same process: 200 steps each, placed and unplaced.
    if args.workload == "llama_7b" and not args.no_other_workloads:
        others = {}
        for name in ("bert_base", "gpt2_medium", "bert_large"):
            ow = W.by_name(name)
            res = {}
            # "on_chip": the same list with the matrices that fit on the on-chip path
            # (came_options.resident; off by default because it measures slower)
            for label, placed, res_mode in (("no_placement", False, resident), ("placed", True, resident),
                                            ("on_chip", False, P.RESIDENT_ON)):
                f, o, _ = run(ow, args.other_steps, 20, placement=placed, resident=res_mode)
                o.close()
                del o
                torch.cuda.empty_cache()
                res[label] = {k: f[k] for k in ("ms_per_step", "value", "bytes_per_param", "whole_step_frac", "bmin_frac",
                                                "streaming_bytes_per_param", "streaming_equivalent_frac",
                                                "on_chip_matrices", "on_chip_elements",
                                                "sweep3_GBs", "phase_ms_per_step", "placement_probe_GBs")}
            res["params"] = ow.n_params
            res["grad_dtype"] = "bf16" if ow.grad_bytes == 2 else "f32"
            res["steps"] = args.other_steps
            others[ow.name] = res
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
