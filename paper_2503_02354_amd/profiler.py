"""Offline performance profiler (paper Section 4.5, "Expert performance metrics"): per architecture, from a
microbenchmark over batch sizes,
  * the execution latency model of Section 4.2, latency(n) = K n + B for a batch of n requests of one expert,
  * the maximum batch size: where the average latency per request has flattened out,
  * the loading latency of an expert (one switch from pinned host memory into the device cache),
and from those the arranging window's thresholds (coe_set_arranging): the group size from which the fixed cost of
running a group now - B, plus the load when the expert is missing - is a small enough share of the whole.

plus the decay-window search of Section 4.4 for the number of experts to keep on the device.

Experts of one architecture are profiled once (Section 4.5).  The measuring functions drive the library through its
binding and need a GPU; the fitting functions are plain arithmetic."""
import math
import time
from typing import Callable, Dict, Sequence, Tuple

import numpy as np


def fit_latency(ns: Sequence[int], us: Sequence[float]) -> Tuple[float, float]:
    """Least-squares line through (n, latency): returns (K, B) in microseconds per request and microseconds."""
    n = np.asarray(ns, np.float64); t = np.asarray(us, np.float64)
    assert n.ndim == 1 and n.shape == t.shape and len(n) >= 2 and np.ptp(n) > 0
    nm, tm = n.mean(), t.mean()
    K = float(((n - nm) * (t - tm)).sum() / ((n - nm) ** 2).sum())
    return K, float(tm - K * nm)


def plateau_batch(ns: Sequence[int], us: Sequence[float], tol: float = 0.05) -> int:
    """The maximum batch size of Section 4.5: the smallest measured batch whose latency per request is within tol of
    the best one measured."""
    per = np.asarray(us, np.float64) / np.asarray(ns, np.float64)
    best = per.min()
    return int(min(n for n, p in zip(ns, per) if p <= best * (1.0 + tol)))


def arranging_window(K_us: float, B_us: float, load_us: float, efficiency: float, max_wait_steps: int) -> Tuple[int, int, int]:
    """Thresholds for coe_set_arranging.  A group of n requests takes K n + B (+ load when its expert is missing); the
    useful share of that is K n / (K n + B [+ load]).  A group is worth running once that share reaches `efficiency`:
    n >= efficiency / (1 - efficiency) * fixed / K.  Returns (min_group_resident, min_group_missing, max_wait_steps)."""
    assert K_us > 0 and 0.0 <= efficiency < 1.0 and B_us >= 0 and load_us >= 0 and max_wait_steps >= 0
    r = efficiency / (1.0 - efficiency)
    return int(math.ceil(r * B_us / K_us)), int(math.ceil(r * (B_us + load_us) / K_us)), int(max_wait_steps)


def experts_for_usage(usage_prob: Sequence[float], percent: float) -> int:
    """Experts sorted by descending usage probability: how many of them it takes to cover `percent` of all usage
    (the CDF of Section 4.4 read from the usage axis to the expert axis); at least one."""
    p = np.sort(np.asarray(usage_prob, np.float64))[::-1]
    cdf = np.cumsum(p) / p.sum() * 100.0
    return int(min(len(p), np.searchsorted(cdf, percent - 1e-9) + 1))


def decay_window_search(usage_prob: Sequence[float], throughput_at: Callable[[int], float], initial_window: float = 20.0,
                        min_points: int = 3, error_margin: float = 0.1, pick: float = 0.5) -> dict:
    """Section 4.4, "Memory allocation under sufficient computation performance": how many experts to keep on the
    device when their memory competes with the memory of large batches.  A window slides up the usage CDF; its first
    size is `initial_window` (percent of all usage) and every slide multiplies the size by the decay factor
    1 - initial_window / 100.  At every position the experts that cover the window's upper bound are loaded and
    `throughput_at(n_experts)` measures sample requests.  A line through the throughputs measured so far predicts the
    next one; the slide stops at the first window whose throughput falls short of the prediction by more than
    `error_margin` (relative), or when every expert is loaded or the next window is too narrow to add one.  The paper then takes any number of experts inside the last window (it
    says a random one: differences inside the window are negligible); `pick` in [0, 1] is that choice, passed in.

    Reading of the paper where it leaves room: the line is fitted through all values measured so far, and the test
    starts once `min_points` values exist.

    Returns dict(n_experts, window=(low %, high %), stopped_by='shortfall' | 'end', trace=[(high %, experts, throughput)])."""
    assert 0.0 < initial_window < 100.0 and min_points >= 2 and 0.0 <= pick <= 1.0
    decay = 1.0 - initial_window / 100.0
    low, size, trace, stopped = 0.0, float(initial_window), [], "end"
    while True:
        high = min(low + size, 100.0)
        n = experts_for_usage(usage_prob, high)
        t = float(throughput_at(n))
        if len(trace) >= min_points:
            K, B0 = fit_latency(range(1, len(trace) + 1), [v[2] for v in trace])      # same least-squares line
            predicted = K * (len(trace) + 1) + B0
            if predicted > 0 and (predicted - t) / predicted > error_margin:
                trace.append((high, n, t))
                stopped = "shortfall"
                break
        trace.append((high, n, t))
        # the window sizes form a geometric series that sums to exactly 100 %: the slide ends when every expert is
        # loaded or the next window is too narrow to add one
        if n >= len(usage_prob) or experts_for_usage(usage_prob, min(high + size * decay, 100.0)) == n:
            break
        low, size = high, size * decay
    return dict(n_experts=experts_for_usage(usage_prob, low + pick * (high - low)), window=(low, high), stopped_by=stopped,
                trace=trace)


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
        ctx.coe_debug_forward(expert_id, n, dev.data_ptr())          # warm-up (first launches, workspace)
        ts = []
        for _ in range(repeats):
            t0 = time.perf_counter()
            ctx.coe_debug_forward(expert_id, n, dev.data_ptr())
            ts.append((time.perf_counter() - t0) * 1e6)
        out[int(n)] = float(np.median(ts))
    return out


def measure_load_latency(B, arch, blob: np.ndarray, repeats: int = 6) -> Dict[str, float]:
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
