"""Offline performance profiler (paper Section 4.5, "Expert performance metrics"): per architecture, from a
microbenchmark over batch sizes,
  * the execution latency model of Section 4.2, latency(n) = K n + B for a batch of n requests of one expert,
  * the maximum batch size: where the average latency per request has flattened out,
  * the loading latency of an expert (one switch from pinned host memory into the device cache),
and from those the arranging window's thresholds (coe_set_arranging): the group size from which the fixed cost of
running a group now - B, plus the load when the expert is missing - is a small enough share of the whole.

Experts of one architecture are profiled once (Section 4.5).  The measuring functions drive the library through its
binding and need a GPU; the fitting functions are plain arithmetic."""
import math
import time
from typing import Dict, Sequence, Tuple

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
