#!/usr/bin/env python3
"""Benchmark of the Adam-mini optimizer step on one MI355X.

A "step" is one pass of the whole hot path -- every launch of adam_mini_step over
the complete tensor list of the workload -- with parameters, first moments,
gradients and v already resident in HBM.  Prints ONE JSON line:
  value       whole-job step throughput in Gparams/s (parameters updated per second / 1e9)
  roofline    dominant kernel: algorithmic bytes per launch / its mean duration measured with
              HIP events on the step's stream during the timed steps, against 8 TB/s
  cpu_baseline  the fp64 CPU oracle timed on a bounded sample of the same workload
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


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--repeats", type=int, default=10,
                    help="timed spans of --steps steps each; ms_per_step is the median span (HIP events)")
    ap.add_argument("--workload", default="llama2_7b",
                    help="tiny | gpt2_small | llama2_7b | llama3_8b | llama2_13b")
    ap.add_argument("--adamw", action="store_true", help="AdamW-equivalent mode: every block of size 1")
    ap.add_argument("--reducer", default="mean", choices=["mean", "norm1", "norm2", "max", "min"],
                    help="block statistic of g*g in the v update (mean = the method; the others are the ablation's)")
    ap.add_argument("--no-bucket-events", action="store_true",
                    help="do not record per-bucket HIP events inside the timed spans (two events per launch distort a "
                         "step of a few microseconds); the roofline then takes each launch's share of the step time")
    ap.add_argument("--allocation", default="arena", choices=["arena", "per-tensor"],
                    help="arena: params, exp_avg and grads are three flat allocations with the tensors back to back "
                         "(each on a 4 KiB boundary), as frameworks with flat parameter and state buffers hold them; "
                         "per-tensor: one allocation per tensor and kind.  Same kernels and launches either way")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other BASELINE configurations (reported under all_configs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="adam_mini_set_option before the layout is built (repeatable)")
    return ap.parse_args()


def traffic_from_profiles(workload: str, kernel: str, with_source: bool = False):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, if there is one.
    It is a figure of that profile run (named by with_source=True: file and the tree it was taken on),
    not something the timed run observes: counters cannot be read from inside the process."""
    rel = os.path.join("profiles", "hbm_traffic_%s.txt" % workload)
    path = os.path.join(ROOT, rel)
    found, tree = None, None
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("# tree:"):
                tree = line.split(":", 1)[1].strip()
            if line.startswith("#") or "=" not in line:
                continue
            kv = dict(tok.split("=", 1) for tok in line.split("\t") if "=" in tok)
            if kv.get("kernel") == kernel and "hbm_bytes_per_launch" in kv:
                found = float(kv["hbm_bytes_per_launch"])
    if with_source:
        return found, (None if found is None else rel + ("@" + tree if tree else ""))
    return found


def time_spans(torch, step_fn, steps, repeats):
    """`repeats` spans of exactly `steps` calls of step_fn each, every span bracketed by a device
    synchronisation on both sides and timed with HIP events on the stream the steps run on (torch's
    current stream) and, beside them, with the host clock.  Returns per-span milliseconds (events)
    and the host-clock figures."""
    ev_ms, host_ms = [], []
    for _ in range(repeats):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        start.record()
        for _ in range(steps):
            step_fn()
        stop.record()
        torch.cuda.synchronize()
        host_ms.append((time.perf_counter() - t0) * 1e3)
        ev_ms.append(start.elapsed_time(stop))
    return ev_ms, host_ms


def median(xs):
    ys = sorted(xs)
    n = len(ys)
    return ys[n // 2] if n % 2 else 0.5 * (ys[n // 2 - 1] + ys[n // 2])


def cpu_baseline(wl, run, hp, target_seconds):
    """Time the oracle (as it stands) on this machine's host cores over a bounded sample: the tensors
    of the first transformer layer, whole, stepped until about target_seconds have been spent."""
    import numpy as np
    import oracle as orc
    from paper_2406_16793_amd.device_state import grad_to_host
    idx = [k for k, s in enumerate(wl.specs) if ".0." in s.name] or list(range(min(4, len(wl.specs))))
    specs = [wl.specs[k] for k in idx]
    st = orc.OracleState([s.numel for s in specs], [s.block_numel for s in specs],
                         [s.wd_scale for s in specs], [run.p[k].cpu().numpy() for k in idx])
    grads = [grad_to_host(run.g[k]) for k in idx]
    ohp = orc.Hyper.from_f32(**hp)
    n = sum(s.numel for s in specs)

    def timed(budget):
        spent, steps = 0.0, 0
        while True:
            t0 = time.perf_counter()
            st.step(grads, ohp)
            dt = time.perf_counter() - t0
            spent += dt
            steps += 1
            if spent + dt > budget or steps >= 2000:
                return steps, spent

    cores = orc.num_threads()
    orc.set_num_threads(1)
    _progress("cpu baseline: oracle on %d tensors" % len(specs))
    steps1, spent1 = timed(0.2 * target_seconds)          # one host thread
    orc.set_num_threads(cores)
    steps, spent = timed(0.8 * target_seconds)            # one thread per host core
    return {"value": n * steps / spent / 1e9, "unit": "Gparams/s", "cores": cores, "kind": "oracle",
            "single_thread_value": n * steps1 / spent1 / 1e9,
            "sample": "%d tensors of layer 0 (%d params, %d blocks); %d oracle steps in %.1f s on %d threads, "
                      "%d steps in %.1f s on 1 thread"
                      % (len(specs), n, sum(s.n_blocks for s in specs), steps, spent, cores, steps1, spent1)}


def _progress(msg):
    """One line per stage on stderr (stdout carries only the JSON line)."""
    sys.stderr.write("[bench] %s\n" % msg)
    sys.stderr.flush()


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
                         "--gpus %d is not supported, use --gpus 1\n" % args.gpus)
        sys.exit(2)
    import torch
    from paper_2406_16793_amd import binding as B
    from paper_2406_16793_amd import partition, workloads
    if not os.path.exists(B.LIB_PATH):
        from paper_2406_16793_amd import build as _build
        _build.build()
    from paper_2406_16793_amd.device_state import DeviceState

    for kv in args.option:
        k, v = kv.split("=", 1)
        B.adam_mini_set_option(k, int(v))
    wl = workloads.get(args.workload)
    if args.adamw:
        wl.specs = partition.as_adamw(wl.specs)
    if args.reducer != "mean":
        wl.specs = partition.with_reducer(wl.specs, args.reducer)
    hp = dict(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay)

    torch.cuda.set_device(0)
    _progress("%s: %d tensors, allocating" % (wl.name, len(wl.specs)))
    run = DeviceState(wl.specs, wl.grad_dtype, arena=args.allocation == "arena")
    for k, s in enumerate(wl.specs):
        run.p[k].copy_(workloads.init_param(s, wl.seed, k, device=run.dev))
        workloads.fill_grad(run.g[k], s, wl, k, 1, row_chunk=8192)
        if k % 64 == 63:
            torch.cuda.synchronize()
            _progress("inputs of %d tensors ready" % (k + 1))
    torch.cuda.synchronize()
    _progress("inputs ready")

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=run.dev)   # 1 GiB
        dst = torch.empty_like(src)
        src.fill_(1.0)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    stream = torch.cuda.current_stream().cuda_stream
    counter = {"t": 0}

    def one_step():
        counter["t"] += 1
        run.opt.step(step=counter["t"], stream=stream, **hp)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    _progress("%d warm-up steps done" % args.warmup)
    # per-bucket HIP events (recorded by the library on the step's stream) stay on during every timed span
    if not args.no_bucket_events:
        B.adam_mini_profile_enable(run.opt.layout, min(4096, args.steps * args.repeats))
    ev_ms, host_ms = time_spans(torch, one_step, args.steps, args.repeats)
    _progress("%d timed spans of %d steps done" % (args.repeats, args.steps))
    buckets = B.adam_mini_profile_read(run.opt.layout)
    B.adam_mini_profile_enable(run.opt.layout, 0)
    # the host clock around a span sees what the events see plus the launch and synchronisation latency;
    # the larger of the two medians is reported, so the figure never undercuts either clock
    span_ms = max(median(ev_ms), median(host_ms))
    elapsed = span_ms * 1e-3

    ms_per_step = elapsed * 1e3 / args.steps
    n_params = sum(s.numel for s in wl.specs)
    n_blocks = run.opt.num_blocks
    gb = 2 if wl.grad_dtype == "bf16" else 4
    per_param = gb + 16 + (8 if args.adamw else 0)

    def algo_bytes(b):
        return b["numel"] * per_param + (0 if args.adamw else 8 * b["n_blocks"])

    if args.no_bucket_events:
        # no per-launch clock: every bucket is charged its share of the step by algorithmic bytes
        total_bytes = sum(algo_bytes(b) for b in buckets)
        for b in buckets:
            b["total_ms"], b["timed_launches"] = ms_per_step * algo_bytes(b) / total_bytes, 1
    dom = max(buckets, key=lambda b: b["total_ms"])
    dom_ms = dom["total_ms"] / max(1, dom["timed_launches"])
    achieved = algo_bytes(dom) / (dom_ms * 1e-3) / 1e9
    traffic, traffic_source = traffic_from_profiles(args.workload + ("_adamw" if args.adamw else ""), dom["kernel"],
                                                    with_source=True)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "kernel": dom["kernel"], "kernel_ms": round(dom_ms, 5),
                "kernel_clock": "share of the step time by algorithmic bytes" if args.no_bucket_events
                else "HIP events recorded by the library around each launch",
                "algorithmic_bytes_per_launch": algo_bytes(dom)}
    whole_gbs = (n_params * per_param + (0 if args.adamw else 8 * n_blocks)) / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "optimizer step Gparams/s + achieved HBM GB/s (% of peak), Llama-2-7B shape",
        "value": round(n_params / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "timing": {"clock": "HIP events on the step's stream, host clock beside them; per span: synchronize, "
                            "%d steps, synchronize" % args.steps,
                   "repeats": args.repeats, "span_ms_median": round(span_ms, 3),
                   "ms_per_step_min": round(min(ev_ms) / args.steps, 4),
                   "ms_per_step_median_events": round(median(ev_ms) / args.steps, 4),
                   "ms_per_step_median_host": round(median(host_ms) / args.steps, 4),
                   "ms_per_step_max": round(max(max(ev_ms), max(host_ms)) / args.steps, 4),
                   "span_at_least_100ms": bool(span_ms >= 100.0)},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name + ("_adamw" if args.adamw else "") + ("" if args.reducer == "mean" else "_" + args.reducer),
                   "params": n_params, "blocks": n_blocks,
                   "tensors": len(wl.specs), "grad_dtype": wl.grad_dtype, "state_dtype": "f32",
                   "allocation": "three flat arenas (params, exp_avg, grads), tensors back to back on 4 KiB boundaries"
                   if args.allocation == "arena" else "one allocation per tensor and kind",
                   "launches_per_step": sum(b["n_kernels"] for b in buckets)},
        "whole_step": {"algorithmic_GBps": round(whole_gbs, 1), "frac_of_peak": round(whole_gbs / HBM_PEAK_GBS, 4),
                       "bytes_per_param": per_param},
        "roofline": roofline,
        "buckets": [{"kernel": b["kernel"], "params": b["numel"], "blocks": b["n_blocks"],
                     "ms": round(b["total_ms"] / max(1, b["timed_launches"]), 4),
                     "GBps": round(algo_bytes(b) / (b["total_ms"] / max(1, b["timed_launches"]) * 1e-3) / 1e9, 1)
                     if b["total_ms"] > 0 else None} for b in buckets],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, run, hp, args.cpu_seconds)
    else:
        out["cpu_baseline"] = None
    run.close()
    del run
    default_run = args.workload == "llama2_7b" and not args.adamw and args.reducer == "mean" and not args.option
    if default_run and not args.no_other_configs:
        arena = args.allocation == "arena"
        # the same workload with the other allocation scheme, so that the effect of the memory layout is on record
        _progress("other allocation scheme: %s" % wl.name)
        other = short_run(torch, workloads, DeviceState, wl.name, not arena)
        if other is not None:
            other["allocation"] = "per-tensor" if arena else "arena"
            out["other_allocation"] = other
        out["all_configs"] = other_configs(out, torch, workloads, DeviceState, arena)
    print(json.dumps(out), flush=True)


def short_run(torch, workloads, DeviceState, name, arena):
    """One workload in the default launch configuration: median of 10 spans of at least 100 ms each.
    None if it does not fit the device."""
    wl = workloads.get(name)
    gb = 2 if wl.grad_dtype == "bf16" else 4
    n_params = sum(s.numel for s in wl.specs)
    if n_params * (8 + gb + 4) + (8 << 30) > torch.cuda.get_device_properties(0).total_memory:
        return None
    torch.cuda.empty_cache()
    run = DeviceState(wl.specs, wl.grad_dtype, arena=arena)
    for k, s in enumerate(wl.specs):
        run.p[k].copy_(workloads.init_param(s, wl.seed, k, device=run.dev))
        workloads.fill_grad(run.g[k], s, wl, k, 1, row_chunk=8192)
    hp = dict(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay)
    stream = torch.cuda.current_stream().cuda_stream
    counter = {"t": 0}

    def one_step():
        counter["t"] += 1
        run.opt.step(step=counter["t"], stream=stream, **hp)

    for _ in range(3):
        one_step()
    est, _ = time_spans(torch, one_step, 3, 1)                      # sizes the spans: at least 100 ms each
    steps = max(3, int(100.0 / max(est[0] / 3, 1e-4)) + 1)
    ev_ms, host_ms = time_spans(torch, one_step, steps, 10)
    ms = max(median(ev_ms), median(host_ms)) / steps
    gbs = (n_params * (16 + gb) + 8 * run.opt.num_blocks) / (ms * 1e-3) / 1e9
    row = {"workload": name, "ms_per_step": round(ms, 5), "Gparams_per_s": round(n_params / ms / 1e6, 2),
           "algorithmic_GBps": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
           "spans": 10, "steps_per_span": steps,
           "ms_per_step_min": round(min(ev_ms) / steps, 5), "ms_per_step_max": round(max(host_ms) / steps, 5)}
    run.close()
    del run
    torch.cuda.empty_cache()
    return row


def other_configs(primary, torch, workloads, DeviceState, arena):
    """Throughput and HBM fraction of every BASELINE configuration on this GPU: the timed workload above plus
    each of the others that fits the device, same launch configuration and allocation scheme."""
    rows = [{"workload": primary["config"]["workload"], "ms_per_step": primary["ms_per_step"],
             "Gparams_per_s": primary["value"], "algorithmic_GBps": primary["whole_step"]["algorithmic_GBps"],
             "frac_of_peak": primary["whole_step"]["frac_of_peak"]}]
    for name in ("tiny", "gpt2_small", "llama3_8b", "llama2_13b"):
        _progress("all_configs: %s" % name)
        row = short_run(torch, workloads, DeviceState, name, arena)
        rows.append(row if row is not None else {"workload": name, "skipped": "does not fit this device"})
    return rows


if __name__ == "__main__":
    main()
