"""Oracle twin of the offline profiler's arithmetic (TEST INFRASTRUCTURE ONLY; plain Python, shares nothing with the library).

Paper Section 4.2: a batch of n requests of one expert takes latency = K n + B.  Section 4.5: K and B are measured
offline; the maximum batch size is where the average latency per request stops falling.  Section 4.4, "Memory allocation
under sufficient computation performance": a window slides along the number of loaded experts; its first size is the
initial window value, every slide multiplies the size by decay factor = 1 - initial window value / 100 (Eq. 1); at every
window as many experts as its upper bound are loaded and sample requests give a throughput; a line f(N) = k N + b through
the first N throughputs (Eq. 2) predicts the next one, and the slide stops when (f(N + 1) - actual) / f(N + 1) exceeds the
error margin (Eq. 3); the number of experts is then taken inside that last window.

Pinned (tests/test_host_logic.py) to the case the paper prints in Section 5.4: initial window 15, error margin 5 %: sizes
15, 12.75, 10.8375, upper bounds 15, 27.75, 38.5875, final window "28 to 39 experts" with a linear error of 7.7 %.
Readings where the paper leaves room: bounds become whole experts by rounding up; the line needs at least two earlier
values (the printed case stops at its third measurement, so two suffice there); the search also ends once a window has
loaded every expert.
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Callable, List, Sequence, Tuple


def line_through(xs: Sequence[float], ys: Sequence[float]) -> Tuple[float, float]:
    """Least-squares slope and intercept from the normal equations, in exact rational arithmetic."""
    X = [Fraction(x) for x in xs]; Y = [Fraction(y) for y in ys]
    n = len(X)
    sx, sy = sum(X), sum(Y)
    sxx = sum(x * x for x in X); sxy = sum(x * y for x, y in zip(X, Y))
    det = n * sxx - sx * sx
    if det == 0:
        raise ValueError("all abscissae equal")
    k = (n * sxy - sx * sy) / det
    b = (sy - k * sx) / n
    return float(k), float(b)


def max_batch(batches: Sequence[int], latency_us: Sequence[float], tol: float) -> int:
    per = [t / n for n, t in zip(batches, latency_us)]
    best = min(per)
    return min(n for n, p in zip(batches, per) if p <= best * (1 + tol))


def arranging_thresholds(k_us: float, b_us: float, load_us: float, efficiency: float) -> Tuple[int, int]:
    """Smallest group sizes n with K n / (K n + fixed) >= efficiency, fixed = B (expert resident) or B + load (missing)."""
    out = []
    for fixed in (b_us, b_us + load_us):
        n = 0
        while k_us * n < efficiency * (k_us * n + fixed) - 1e-12 * (k_us * n + fixed):
            n += 1
        out.append(n)
    return out[0], out[1]


def window_bounds(initial_window: float, k: int) -> Tuple[float, float]:
    """Bounds of window k on the expert axis."""
    decay = 1 - initial_window / 100
    low = sum(initial_window * decay ** i for i in range(k))
    return low, low + initial_window * decay ** k


def whole(bound: float, total: int) -> int:
    return max(1, min(total, math.ceil(bound - 1e-9)))


def decay_window_search(total: int, throughput_at: Callable[[int], float], initial_window: float, error_margin: float,
                        fit_points: int = 2) -> dict:
    """Runs the whole search, calling throughput_at(number of experts) once per window.  Returns dict(window=(low, high),
    experts=(n_low, n_high), stopped_by='shortfall' | 'end', linear_error, loaded=[...], throughputs=[...])."""
    ts: List[float] = []
    loaded: List[int] = []
    k = 0
    while True:
        low, high = window_bounds(initial_window, k)
        n = whole(high, total)
        t = float(throughput_at(n))
        err = 0.0
        if len(ts) >= fit_points:
            slope, icpt = line_through(range(1, len(ts) + 1), ts)
            predicted = slope * (len(ts) + 1) + icpt
            if predicted > 0:
                err = (predicted - t) / predicted
        ts.append(t); loaded.append(n)
        if err > error_margin:
            stopped = "shortfall"
            break
        if n >= total:
            stopped = "end"
            break
        k += 1
    return dict(window=(low, high), experts=(whole(low, total), whole(high, total)), stopped_by=stopped, linear_error=err,
                loaded=loaded, throughputs=ts)


def memory_scores(nbytes: Sequence[int]) -> Tuple[list, int]:
    """Section 4.5: memory footprints normalised to memory scores; the unit is the smallest footprint."""
    unit = min(nbytes)
    return [b / unit for b in nbytes], unit


def expert_budget(total_bytes: int, reserve_bytes: int, bytes_per_request: int, max_batch: int) -> int:
    """Section 4.4, limited computation performance: inference gets the memory of the maximum batch, experts the rest."""
    return max(0, total_bytes - reserve_bytes - bytes_per_request * max_batch)


def executable_batch(free_bytes: int, bytes_per_request: int, profiled_max_batch: int) -> int:
    """Section 4.2 "Request splitting": the smaller of what memory holds and what the profiler measured."""
    return min(free_bytes // bytes_per_request, profiled_max_batch)


def usage_probabilities(paths, n_experts: int):
    """Section 4.5 "Expert information": share of the sampled requests whose path visits each expert (paths: rows of
    expert ids, -1 padded)."""
    n = len(paths)
    visits = [0] * n_experts
    for p in paths:
        for e in set(int(v) for v in p if v >= 0):
            visits[e] += 1
    return [v / n for v in visits]
