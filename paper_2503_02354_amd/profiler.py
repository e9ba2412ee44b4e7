"""Offline performance profiler (paper Section 4.5, "Expert performance metrics"; Section 4.4 memory allocation): the
measuring side.  It drives the library through its binding on a GPU - forwards over batch sizes, expert switches, sample
passes with a given number of resident experts - and hands the numbers to the library's profiler arithmetic
(coe_profiler_* in include/coe.h): the latency model K n + B of Section 4.2, the maximum batch size, the arranging window's
thresholds and the decay-window search for the number of experts to keep on the device.  Experts of one architecture are
profiled once (Section 4.5).  No arithmetic of the method lives here."""
import time
from typing import Callable, Dict, Sequence, Tuple

import numpy as np

from . import binding as B


def measure_batch_latency(ctx, expert_id: int, in_shape: Tuple[int, int, int], sizes: Sequence[int], repeats: int = 3,
                          dtype=np.uint16) -> Dict[int, float]:
    """Median wall-clock latency in microseconds of one forward of `expert_id` over n inputs, for each n in sizes
    (inputs resident on the device; the call returns when the logits are back on the host)."""
    import torch
    h, w, c = in_shape
    nmax = max(sizes)
    rng = np.random.default_rng(0)
    if dtype == np.uint16:
        x = (rng.standard_normal((nmax, h, w, c)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
        dev = torch.from_numpy(x.view(np.int16)).cuda()
    else:
        dev = torch.from_numpy(rng.standard_normal((nmax, h, w, c)).astype(np.float32)).cuda()
    out = {}
    for n in sizes:
        ctx.coe_debug_forward(expert_id, n, dev.data_ptr())          # warm-up (first launches)
        ts = []
        for _ in range(repeats):
            t0 = time.perf_counter()
            ctx.coe_debug_forward(expert_id, n, dev.data_ptr())
            ts.append((time.perf_counter() - t0) * 1e6)
        out[int(n)] = float(np.median(ts))
    return out


def measure_load_latency(arch, blob: np.ndarray, repeats: int = 6) -> Dict[str, float]:
    """Loading latency of one expert of `arch`: two experts share a one-expert cache and requests alternate between
    them, so every step is a switch; the copy-stream events around the copies give the time.  Returns
    dict(us=..., GBps=..., bytes=...)."""
    import torch
    ctx = B.Context(max_requests=4, max_stages=1, max_batch=4, cache_cap_experts=1, profile=1)
    try:
        aid = ctx.coe_register_arch(arch)
        for e in range(2):
            ctx.coe_register_expert(e, aid, blob, 0.5)
        ctx.coe_set_dependency_graph(np.zeros(3, np.int32), np.zeros(0, np.int32))
        x = torch.zeros((1, arch.in_h, arch.in_w, arch.in_c), dtype=torch.int16 if arch.dtype == 1 else torch.float32).cuda()
        k_switch = B.KERNEL_CLASS_NAMES.index("switch")
        for i in range(repeats + 2):
            if i == 2:
                ctx.coe_sync(); ctx.coe_profile_read(k_switch)       # drop the initial fill and the first switch
            ctx.coe_submit(1, x.data_ptr(), True, np.array([i % 2], np.int32))
            ctx.coe_step()
            ctx.coe_collect(4)
        ctx.coe_sync()
        launches, ms, work = ctx.coe_profile_read(k_switch)
        assert launches > 0, "no switch was timed"
        us = ms * 1e3 / launches
        return dict(us=us, GBps=work / launches / us / 1e3, bytes=work / launches)
    finally:
        ctx.close()


def profile_arch(arch, blob: np.ndarray, sizes: Sequence[int], max_batch: int, efficiency: float = 0.2, tol: float = 0.05,
                 repeats: int = 3) -> dict:
    """Everything Section 4.5 lists for one architecture, measured on this GPU: K and B of the latency model (fit over
    `sizes`), the maximum batch size among `sizes`, the load latency, and the arranging thresholds that follow.  Returns
    dict(K_us, B_us, load_us, load_GBps, max_batch, min_group_resident, min_group_missing, latency_us={n: us})."""
    ctx = B.Context(max_requests=max(sizes), max_stages=1, max_batch=max_batch)
    try:
        aid = ctx.coe_register_arch(arch)
        ctx.coe_register_expert(0, aid, blob, 1.0)
        ctx.coe_set_dependency_graph(np.zeros(2, np.int32), np.zeros(0, np.int32))
        lat = measure_batch_latency(ctx, 0, (arch.in_h, arch.in_w, arch.in_c), sizes, repeats,
                                    np.uint16 if arch.dtype == 1 else np.float32)
    finally:
        ctx.close()
    ns = sorted(lat)
    K, Bc = B.coe_profiler_fit_latency(ns, [lat[n] for n in ns])
    load = measure_load_latency(arch, blob)
    lo, hi = B.coe_profiler_arranging_window(max(K, 1e-9), max(Bc, 0.0), load["us"], efficiency)
    return dict(K_us=K, B_us=Bc, load_us=load["us"], load_GBps=load["GBps"], max_batch=B.coe_profiler_max_batch(ns, [lat[n] for n in ns], tol),
                min_group_resident=lo, min_group_missing=hi, latency_us=lat)


def search_resident_experts(n_experts_total: int, throughput_at: Callable[[int], float], initial_window: float = 15.0,
                            error_margin: float = 0.05, fit_points: int = 2) -> dict:
    """The decay-window search of Section 4.4 with measured throughputs: throughput_at(n) loads the n most used experts,
    runs sample requests and returns the throughput.  The window arithmetic is the library's (coe_profiler_window_step).
    Returns dict(window=(low, high), experts=(n_low, n_high), stopped_by, linear_error, loaded=[...], throughputs=[...])."""
    ts, loaded = [], []
    st = B.coe_profiler_window_step(n_experts_total, initial_window, error_margin, fit_points, ts)
    while st.status == B.COE_WINDOW_MEASURE:
        loaded.append(st.n_next)
        ts.append(float(throughput_at(st.n_next)))
        st = B.coe_profiler_window_step(n_experts_total, initial_window, error_margin, fit_points, ts)
    return dict(window=(st.window_low, st.window_high), experts=(st.n_low, st.n_high),
                stopped_by="shortfall" if st.status == B.COE_WINDOW_SHORTFALL else "end", linear_error=st.linear_error,
                loaded=loaded, throughputs=ts)
