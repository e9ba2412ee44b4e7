#!/usr/bin/env python3
"""Benchmark of the CoE hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic requests: coe_submit (inputs already in
HBM) -> coe_step per stage (regroup, split, cache, expert forwards, routing) -> coe_collect.
Workload = 16 ResNet-18-shaped bf16 experts, 4096 requests of 3x224x224, two-stage tree, all experts resident.

Prints ONE JSON line: requests/s plus a roofline object for the dominant kernel (the bf16 MFMA implicit-GEMM
convolution, timed with HIP events on the library's compute stream over the timed region) and the CPU oracle timed
on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
# HBM bytes per launch of conv3x3_slab_kernel on this workload, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE)
# scaled by what the same counters read for the gather kernel's plain copy (profiles/conv3x3_slab_config2_hbm_counters.md).
# Tied to the kernel source and the launch configuration it was measured on: an edit of that file, another workload,
# batch cap or grouping threshold make bench.py report null again.
SLAB_TRAFFIC_BYTES_PER_LAUNCH = 2329.8e6
SLAB_TRAFFIC_SOURCE = ("paper_2503_02354_amd/csrc/conv_mfma.hip",
                       "da23a53c7c541e6dd6397032f79f58e0a921a3f097e18b8be3344e87c0625597")
SLAB_TRAFFIC_LAUNCH_CONFIG = ("config2", 0, 4096, 512, 1, "")   # workload, requests, max_batch, group_small, arrivals per step, window


def measured_traffic(kernel: str, launch_config=None):
    if kernel != "conv3x3_slab_kernel" or launch_config != SLAB_TRAFFIC_LAUNCH_CONFIG:
        return None
    import hashlib
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), SLAB_TRAFFIC_SOURCE[0])
    try:
        with open(path, "rb") as f:
            same = hashlib.sha256(f.read()).hexdigest() == SLAB_TRAFFIC_SOURCE[1]
    except OSError:
        same = False
    return SLAB_TRAFFIC_BYTES_PER_LAUNCH if same else None
PEAK_HBM_GBS = 8000.0


def arch_macs(arch) -> int:
    """Multiply-accumulates of one request through the expert (conv, FC and attention contractions)."""
    import coe_workloads as W
    total = 0
    for L, (sshape, dshape) in zip(arch.layers, W.walk(arch)):
        op, k, r, s = int(L[0]), int(L[4]), int(L[5]), int(L[6])
        h, w, c = sshape
        if op == W.OP_CONV:
            total += dshape[0] * dshape[1] * k * r * s * c
        elif op in (W.OP_HEAD, W.OP_HEAD_CLS):
            total += k * c
        elif op == W.OP_ATTENTION:
            d = c // 3
            total += 2 * h * h * d
    return total


WORKLOAD_TEXT = {
    "config2": "config2: 16 ResNet-18-shaped bf16 experts, 4096 requests 3x224x224, 2-stage tree (1 root -> 15 leaves), "
               "all resident",
    "config3": "config3: 64 ResNet-50-shaped bf16 experts, 16384 requests 3x224x224 arriving in batches of 512, 2-stage tree "
               "(1 root -> 63 leaves, Zipf(1.1) usage), device cache capped at 16 experts",
    "config4": "config4: 120 mixed ResNet-18/ResNet-50-shaped bf16 experts in a 3-stage DAG with shared downstream experts, "
               "8192 requests 3x224x224 with skewed group sizes, all resident",
    "config5": "config5: 32 ViT-B/16-shaped bf16 experts, 4096 requests 3x224x224, 2-stage tree (1 root -> 31 leaves, uniform "
               "usage), device cache capped at 12 experts",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="config2", choices=["config2", "config3", "config4", "config5"],
                    help="config2 (default) is the benchmark line; config3 / config5 have a capped expert cache and report "
                         "switch bandwidth, overlap and host planning time next to their throughput")
    ap.add_argument("--requests", type=int, default=0, help="0 = the workload's own request count")
    ap.add_argument("--max-batch", type=int, default=0,
                    help="most requests per launch sequence (0 = 4096 for config2 / config4, where 288 GB of HBM hold the "
                         "activations of a whole stage and large launches fill whole rounds of compute units; 512 otherwise)")
    ap.add_argument("--cpu-sample", type=int, default=384, help="requests the oracle is timed on (0 = skip)")
    ap.add_argument("--arrivals-per-step", type=int, default=1,
                    help="arrival batches that queue up between two stages (1: a stage after every arrival, the least "
                         "favourable case; more: later arrivals join the groups of earlier ones before they run, which is "
                         "what request arranging is for)")
    ap.add_argument("--group-small", type=int, default=None,
                    help="groups of at most this many requests share launches (default: 512 for config2 / config4, so the "
                         "leaf groups of a stage run as one launch per layer; otherwise 0 = the library's default; -1 = never)")
    ap.add_argument("--arrange", default="",
                    help="arranging window 'min_resident,min_missing,max_wait' for every architecture: a queued group "
                         "smaller than min_resident (expert on the device) or min_missing (expert missing) waits up to "
                         "max_wait steps for later arrivals to join it.  Default: '0,43,8' for config3 (requests arrive in "
                         "512-request batches there; 43 is where the offline profiler puts a missing ResNet-50 group at "
                         "20 %% efficiency), off elsewhere; 'off' = every queued group runs in every step")
    ap.add_argument("--eviction", default="two-stage", choices=["two-stage", "lru", "fifo"],
                    help="replacement rule of the expert cache: the paper's two-stage rule (default) or the rules of the "
                         "systems it compares with")
    ap.add_argument("--prefetch-depth", type=int, default=-1,
                    help="experts of this many groups right before a missing one in the plan count as in use while its copy "
                         "is in flight (0: consecutive misses reuse one slot and each copy waits for the group before it).  "
                         "Default: 4 for config3, 2 for config5 (the workloads with a capped cache), 0 elsewhere")
    ap.add_argument("--executors", type=int, default=0,
                    help="executors: launch sequences of different groups run on this many streams (1-3); the kernels of "
                         "small groups then overlap on the device.  Default: 3 for config3 (many small groups per step), "
                         "1 elsewhere: per-launch rates in `roofline` drop when kernels share the chip, and the large "
                         "launches of the other workloads gain 0-3 %%")
    ap.add_argument("--no-profile", action="store_true", help="do not time kernel classes with events")
    ap.add_argument("--profile-every", type=int, default=0,
                    help="time every k-th launch of each kernel class (0 = every launch for config2 / config4, whose steps "
                         "are a few dozen large launches; 7 otherwise: an event pair costs a pipeline bubble, and 7 is "
                         "coprime to the launches per forward, so every layer shape is sampled)")
    args = ap.parse_args()
    big = args.workload in ("config2", "config4")
    if args.max_batch == 0:
        args.max_batch = 4096 if big else 512
    if args.group_small is None:
        args.group_small = 512 if big else 0
    if args.profile_every == 0:
        args.profile_every = 1 if args.workload == "config2" else 7
    if args.arrange == "":
        args.arrange = "0,43,8" if args.workload == "config3" else "off"
    if args.arrange == "off":
        args.arrange = ""
    if args.executors == 0:
        args.executors = 3 if args.workload == "config3" else 1
    if args.prefetch_depth < 0:
        args.prefetch_depth = {"config3": 4, "config5": 2}.get(args.workload, 0)
    if args.gpus != 1:
        print("bench.py runs on exactly one GPU: the library has no multi-GPU path (--gpus 1 only)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    from paper_2503_02354_amd import binding as B
    import coe_workloads as W

    make = {"config2": W.config2, "config3": W.config3, "config4": W.config4, "config5": W.config5}[args.workload]
    wl = make(args.requests) if args.requests else make()
    n = wl.n_requests
    arch = wl.archs[0]
    t0 = time.time()
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(8) as ex:
        blobs = list(ex.map(wl.blob, range(wl.graph.n_experts)))
    x = wl.inputs(range(n))
    t_gen = time.time() - t0

    ctx = B.Context(max_requests=n, max_stages=wl.max_stages, max_batch=args.max_batch,
                    cache_cap_experts=wl.cache_cap_experts, profile=0 if args.no_profile else args.profile_every,
                    group_small=args.group_small, eviction=["two-stage", "lru", "fifo"].index(args.eviction), prefetch_depth=args.prefetch_depth, executors=args.executors)
    B.setup_workload(ctx, wl, blobs)
    # latency models from the offline profiler on this GPU (ns per request, ns per launch sequence, ns per expert load)
    LATENCY = {"resnet18": (3830, 886000, 408000), "resnet50": (14410, 1611000, 846000)}
    for a, arch_a in enumerate(wl.archs):
        if arch_a.name in LATENCY:
            ctx.coe_set_latency_model(a, *LATENCY[arch_a.name])
    window = [int(v) for v in args.arrange.split(",")] if args.arrange else None
    if window:
        assert len(window) == 3, "--arrange takes min_resident,min_missing,max_wait"
        for a in range(len(wl.archs)):
            ctx.coe_set_arranging(a, *window)
    dev = torch.from_numpy(x.view(np.int16)).cuda()
    torch.cuda.synchronize()

    per = x[0].nbytes
    arrival = wl.arrival_batch or n
    step_stats = []

    def one_step():
        # requests arrive in batches of `arrival`; every arrival is followed by one stage over everything pending
        steps_run = 0
        for k, s0 in enumerate(range(0, n, arrival)):
            m = min(arrival, n - s0)
            ctx.coe_submit(m, dev.data_ptr() + s0 * per, True, None if wl.first_expert is None else wl.first_expert[s0:s0 + m])
            if (k + 1) % max(args.arrivals_per_step, 1) and s0 + arrival < n:
                continue
            rc, st = ctx.coe_step()
            step_stats.append(st)
            steps_run += 1
        # without a window the graph's depth bounds the steps left (no empty probing step after them); with one, groups
        # may still be waiting: step until the queue is empty
        for _ in range(wl.max_stages - 1 if not window else 10 ** 6):
            rc, st = ctx.coe_step()
            if rc == B.COE_DONE:
                break
            step_stats.append(st)
        ids, logits, path = ctx.coe_collect(n)
        assert len(ids) == n, f"only {len(ids)} of {n} requests finished"
        order = np.argsort(ids)
        return path[order]

    for _ in range(args.warmup):
        path = one_step()
    ctx.coe_sync()
    for k in range(len(B.KERNEL_CLASS_NAMES)):
        ctx.coe_profile_read(k)            # drop warm-up spans
        ctx.coe_profile_issued(k)
    torch.cuda.synchronize()
    step_stats.clear()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        path = one_step()
    ctx.coe_sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / max(args.steps, 1)
    value = n * args.steps / elapsed

    prof = {}
    if not args.no_profile:
        for k, name in enumerate(B.KERNEL_CLASS_NAMES):
            launches, ms, work = ctx.coe_profile_read(k)
            issued = ctx.coe_profile_issued(k)
            if launches:
                prof[name] = {"launches": launches, "ms": round(ms, 3), "work": work, "issued": issued}
    # (FLOPs of the experts every request actually visited, from the collected paths)
    macs_of = [arch_macs(wl.archs[wl.expert_arch[e]]) for e in range(wl.graph.n_experts)]
    # the matrix-core convolution classes; the roofline object is for the one that takes the most time
    mfma_kernels = {"conv_slab": "conv3x3_slab_kernel", "conv_mfma": "conv_igemm_dma_kernel", "attention": "attention_kernel"}
    est_ms = {name: prof[name]["ms"] / prof[name]["launches"] * prof[name]["issued"] for name in mfma_kernels if name in prof}
    roofline = None
    if est_ms:
        dom = max(est_ms, key=est_ms.get)
        p = prof[dom]
        achieved = p["work"] / (p["ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": mfma_kernels[dom], "achieved": round(achieved, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic(mfma_kernels[dom], (args.workload, args.requests, args.max_batch, args.group_small,
                                                                              args.arrivals_per_step, args.arrange)),
                    "traffic_unit": "HBM bytes per launch",
                    "launches_timed": p["launches"], "launches": p["issued"],
                    "avg_launch_us": round(p["ms"] * 1e3 / p["launches"], 2),
                    "share_of_step": round(est_ms[dom] / args.steps / ms_per_step, 3)}
    other = {}
    for name in ("conv_slab", "conv_mfma", "attention", "token_ops", "regroup_gather", "switch", "pool", "conv_stem",
                 "conv_direct", "head", "regroup_index"):
        if name in prof:
            p = prof[name]
            # timed launches are every k-th of the class: scale their mean to all launches
            entry = {"ms_per_step": round(p["ms"] / p["launches"] * p["issued"] / args.steps, 3),
                     "launches_per_step": p["issued"] // max(args.steps, 1)}
            if name in ("regroup_gather", "pool", "switch", "token_ops"):
                entry["GB/s"] = round(p["work"] / (p["ms"] * 1e-3) / 1e9, 1) if p["ms"] > 0 else None
            if name in ("conv_direct", "conv_stem", "conv_slab", "conv_mfma", "attention"):
                entry["TFLOP/s"] = round(p["work"] / (p["ms"] * 1e-3) / 1e12, 2)
            other[name] = entry

    leaves = np.bincount(path[:, 1][path[:, 1] >= 0], minlength=wl.graph.n_experts)[1:]
    visits = np.bincount(path[path >= 0].ravel(), minlength=wl.graph.n_experts)
    flops_per_step = 2.0 * float(np.dot(visits, macs_of))

    # expert cache: switches of the timed region (copy-stream events bracket every H2D copy) and the host planning time
    cache = None
    if step_stats:
        misses = sum(st.n_misses for st in step_stats)
        cache = {"cap_experts": wl.cache_cap_experts, "replacement": args.eviction, "prefetch_depth": args.prefetch_depth, "switches_per_pass": misses // max(args.steps, 1),
                 "evictions_per_pass": sum(st.n_evictions for st in step_stats) // max(args.steps, 1),
                 "bytes_switched_per_pass": sum(st.bytes_switched for st in step_stats) // max(args.steps, 1),
                 "host_plan_us_per_step": round(float(np.mean([st.host_plan_us for st in step_stats])), 1)}
        if "switch" in prof:
            sw = prof["switch"]
            copy_ms = sw["ms"] / sw["launches"] * sw["issued"] / args.steps
            cache["switch_GB/s"] = round(sw["work"] / (sw["ms"] * 1e-3) / 1e9, 1)
            cache["copy_ms_per_pass"] = round(copy_ms, 2)
            cache["copy_share_of_pass"] = round(copy_ms / ms_per_step, 3)

    cpu = None
    if args.cpu_sample > 0:
        from oracle import oracle as O
        m = min(args.cpu_sample, n)
        t0 = time.perf_counter()
        ref = O.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, x[:m], None, wl.max_stages,
                          wl.max_classes)
        dt = time.perf_counter() - t0
        agree = float(np.mean((ref["path"] == path[:m]).all(axis=1)))
        cpu = {"value": round(m / dt, 3), "unit": "requests/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"first {m} requests of the same workload, full {wl.max_stages}-stage chain, {dt:.1f}s",
               "route_agreement_unguarded": round(agree, 4)}

    out = {
        "metric": "requests/s through a multi-stage CoE chain (1 GPU)", "value": round(value, 1), "unit": "requests/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "requests": n, "arrival_batch": arrival,
                   "arrivals_per_step": args.arrivals_per_step, "max_batch": args.max_batch, "executors": args.executors,
                   "arranging_window": None if not window else {"min_group_resident": window[0], "min_group_missing": window[1],
                                                                "max_wait_steps": window[2]},
                   "stages": wl.max_stages, "gflop_per_request": round(flops_per_step / n / 1e9, 3)},
        "end_to_end_tflops": round(flops_per_step / (ms_per_step * 1e-3) / 1e12, 2),
        "end_to_end_frac_of_bf16_peak": round(flops_per_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline, "kernel_classes": other, "expert_cache": cache,
        "grouped_launches": None if not step_stats else {
            "groups_per_pass": sum(st.n_groups for st in step_stats) // max(args.steps, 1),
            "of_them_in_shared_launches": sum(st.n_grouped for st in step_stats) // max(args.steps, 1),
            "shared_launch_sequences": sum(st.n_group_sets for st in step_stats) // max(args.steps, 1)},
        "arranging": None if not (step_stats and window) else {
            "steps_per_pass": len(step_stats) // max(args.steps, 1),
            "group_waits_per_pass": sum(st.n_deferred_groups for st in step_stats) // max(args.steps, 1),
            "request_waits_per_pass": sum(st.n_deferred_requests for st in step_stats) // max(args.steps, 1)},
        "cpu_baseline": cpu,
        "leaf_group_sizes": {"min": int(leaves.min()), "max": int(leaves.max())},
        "input_generation_s": round(t_gen, 1),
        "paper_context": "the paper reports 4.5x-12x throughput over prior systems (Samba-CoE variants) on an RTX 3080Ti/"
                         "Xeon Silver 4214R box and an Apple M2 - context only",
    }
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
