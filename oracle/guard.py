"""Oracle-side workload preparation (TEST INFRASTRUCTURE ONLY; calls the oracle and the input generators, never the HIP path).

* margin guard: a float argmax is only well posed away from ties, so a request whose oracle top-2 gap at any routing
  stage is below delta * (largest computed logit magnitude) is re-drawn from its next sub-seed; both sides then see
  the same re-drawn input.
* head-bias calibration: random-weight experts on noise images give nearly identical logits for every request, so
  the routing experts' head biases are offset (from oracle logits only) until the routed classes follow a target
  distribution.  The offsets are inputs to both sides.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from . import oracle as O

# Smallest admissible top-2 gap at a routing stage, as a fraction of the largest |logit - head bias| of that expert (the
# part of the logit that is computed; the head bias is added exactly and calibrated biases cancel most of the logit, so
# the final logit's magnitude says nothing about the arithmetic noise on it).
#
# Where the numbers come from: the HIP path accumulates in fp32 in another order than the oracle's fp64, which now and then
# flips the bf16 rounding of a stored activation; the flips of all layers add up to a logit difference eps, measured on the
# GPU against this oracle over 512 unfiltered requests per full-size workload (tests/test_gpu_full_size.py prints the
# census and fails if it outgrows these constants): eps <= 3.1e-3 of the computed magnitude for the ResNet-shaped experts
# (20-53 stored layers, logits dominated by a common positive part), eps <= 2.1e-2 for the ViT-B/16-shaped ones (~100
# stored tensors per forward, and a head over layer-normalised features whose logits are a cancelling sum as large as the
# noise of 30 features).  Two logits can move towards each other by 2 eps, so the argmax is decidable when the gap
# exceeds 2 eps; delta = 2.5 to 3 eps.  fp32 experts: only the fp32 summation order differs.
DELTA_CNN_BF16 = 8e-3
DELTA_VIT_BF16 = 6e-2
DELTA_F32 = 1e-4


def delta_for_arch(arch) -> float:
    if arch.dtype != 1:
        return DELTA_F32
    return DELTA_VIT_BF16 if arch.name == "vit" else DELTA_CNN_BF16


def delta_for(wl) -> float:
    """Largest delta over the workload's architectures (a single conservative figure for reports)."""
    return max(delta_for_arch(a) for a in wl.archs)


def _head_bias(wl, blobs, e, cache):
    import coe_workloads as W
    if e not in cache:
        a = wl.archs[wl.expert_arch[e]]
        cache[e] = W.blob_tensor(a, blobs[e], a.n_layers - 1, "b")
    return cache[e]


def routing_margins(wl, blobs, res, delta: Optional[float] = None) -> np.ndarray:
    """[n][max_stages]: (top1 - top2 over the routed classes) / max_c |logit_c - bias_c| at every routing stage a request
    went through, divided by that expert's delta (so values below 1 are undecidable), -1 elsewhere."""
    n, S = res["path"].shape
    out = np.full((n, S), -1.0)
    bias_cache = {}
    for r in range(n):
        for s in range(S):
            e = int(res["path"][r, s])
            if e < 0:
                break
            k = int(wl.graph.succ_off[e + 1] - wl.graph.succ_off[e])
            if k == 0:
                break
            b = _head_bias(wl, blobs, e, bias_cache)
            lg = res["all_logits"][r, s, :len(b)].astype(np.float64)
            scale = max(np.abs(lg - b).max(), 1e-30)
            top = np.sort(lg[:k])[::-1]
            d = delta if delta is not None else delta_for_arch(wl.archs[wl.expert_arch[e]])
            out[r, s] = (top[0] - top[1]) / scale / d if k > 1 else 1e30
    return out


# progress(done, total) is called between pieces of a long oracle run, if set (long runs on a box that takes silence for a hang)
PROGRESS = None
PIECE = 64


def run(wl, blobs, inputs, first_expert=None, threads: int = 0):
    n = len(inputs)
    if PROGRESS is None or n <= PIECE:
        return O.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, inputs, first_expert,
                           wl.max_stages, wl.max_classes, threads)
    parts = []
    for s0 in range(0, n, PIECE):
        fe = None if first_expert is None else first_expert[s0:s0 + PIECE]
        parts.append(O.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, inputs[s0:s0 + PIECE], fe,
                                 wl.max_stages, wl.max_classes, threads))
        PROGRESS(min(s0 + PIECE, n), n)
    return {k: np.concatenate([p[k] for p in parts]) for k in parts[0]}


def guarded_inputs(wl, blobs, request_ids: Sequence[int], delta: Optional[float] = None, max_rounds: int = 8):
    """Returns (inputs, subseeds, oracle_result, n_redraws) for the given request ids.  oracle_result["ambiguous"] marks
    the requests that still have a routing gap below delta after max_rounds re-draws: for those the admissible outcomes
    are enumerated with admissible_outcomes().  oracle_result["first_draw"] keeps the path and the per-stage logits of
    the unfiltered first draw (sub-seed 0) of every request, for censuses over an unfiltered population.
    delta None = every expert's own (delta_for_arch)."""
    ids = np.asarray(list(request_ids), dtype=np.int64)
    sub = np.zeros(len(ids), np.int32)
    x = wl.inputs(ids, sub)
    fe = None if wl.first_expert is None else wl.first_expert[ids]
    res = run(wl, blobs, x, fe)
    first = dict(path=res["path"].copy(), all_logits=res["all_logits"].copy())
    redraws = 0
    bad = np.zeros(0, dtype=np.int64)
    for rnd in range(max_rounds + 1):
        m = routing_margins(wl, blobs, res, delta)
        bad = np.nonzero(((m >= 0) & (m < 1.0)).any(axis=1))[0]
        if rnd == 0:
            first["undecidable"] = ((m >= 0) & (m < 1.0)).any(axis=1)
        if len(bad) == 0 or rnd == max_rounds:
            break
        redraws += len(bad)
        sub[bad] += 1
        x[bad] = wl.inputs(ids[bad], sub[bad])
        r2 = run(wl, blobs, x[bad], None if fe is None else fe[bad])
        for k in res:
            res[k][bad] = r2[k]
    amb = np.zeros(len(ids), bool)
    amb[bad] = True
    res["ambiguous"] = amb
    res["first_draw"] = first
    return x, sub, res, redraws


def evaluate_pairs(wl, blobs, xs: np.ndarray, experts: Sequence[int], threads: int = 0) -> np.ndarray:
    """Oracle logits of expert experts[i] on input xs[i], all pairs in parallel (a graph without routes makes the
    chain runner evaluate exactly the first expert of every request)."""
    E = wl.graph.n_experts
    experts = np.asarray(experts, np.int32)
    out = []
    piece = PIECE if PROGRESS is not None else max(len(xs), 1)
    for s0 in range(0, len(xs), piece):
        r = O.run_chain(wl.archs, wl.expert_arch, blobs, np.zeros(E + 1, np.int32), np.zeros(1, np.int32), xs[s0:s0 + piece],
                        experts[s0:s0 + piece], 1, wl.max_classes, threads)
        out.append(r["logits"])
        if PROGRESS is not None and len(xs) > piece:
            PROGRESS(min(s0 + piece, len(xs)), len(xs))
    return np.concatenate(out) if out else np.zeros((0, wl.max_classes), np.float32)


def admissible_outcomes_batch(wl, blobs, xs: np.ndarray, first_experts: Sequence[int], delta: Optional[float] = None):
    """For every request: every outcome that is correct up to the routing tolerance.  At each routing stage every class
    whose logit is within delta * (largest computed logit magnitude) of the maximum may be taken.  Returns one list per
    request of (path [max_stages] int32, final logits [max_classes] float32), in no particular order."""
    n = len(xs)
    done = [[] for _ in range(n)]
    frontier = [(i, int(first_experts[i]), []) for i in range(n)]        # (request, expert to run, path so far)
    bias_cache = {}
    while frontier:
        lg_all = evaluate_pairs(wl, blobs, xs[[f[0] for f in frontier]], [f[1] for f in frontier])
        nxt_frontier = []
        for (i, e, path), lg in zip(frontier, lg_all):
            path = path + [e]
            succ = wl.graph.successors(e)
            k = len(succ)
            if k == 0:
                done[i].append((path, lg)); continue
            b = _head_bias(wl, blobs, e, bias_cache)
            scale = max(float(np.abs(lg[:len(b)].astype(np.float64) - b).max()), 1e-30)
            d = delta if delta is not None else delta_for_arch(wl.archs[wl.expert_arch[e]])
            order = np.argsort(-lg[:k], kind="stable")
            for c in order:
                if lg[order[0]] - lg[c] > d * scale:
                    break
                nxt = int(succ[c])
                if nxt == -1:
                    done[i].append((path, lg))
                else:
                    nxt_frontier.append((i, nxt, path))
        frontier = nxt_frontier
    out = []
    for i in range(n):
        res = []
        for path, lg in done[i]:
            p = np.full(wl.max_stages, -1, np.int32); p[:len(path)] = path
            res.append((p, np.asarray(lg, np.float32)))
        out.append(res)
    return out


def admissible_outcomes(wl, blobs, x_r: np.ndarray, first_expert: int = 0, delta: Optional[float] = None):
    """Single-request form of admissible_outcomes_batch."""
    return admissible_outcomes_batch(wl, blobs, x_r[None], [first_expert], delta)[0]


def calibrate_bias(z: np.ndarray, n_route: int, target: np.ndarray, iters: int = 400, lr: float = 0.5) -> np.ndarray:
    """z: [n][classes] oracle logits with zero head bias.  Returns a bias [classes] such that argmax over the first
    n_route classes of z + bias follows `target` (length n_route) as closely as the sample allows."""
    n, ncls = z.shape
    zr = z[:, :n_route].astype(np.float64)
    scale = max(zr.std(axis=0).mean(), 1e-12)
    b = -zr.mean(axis=0)
    tgt = np.asarray(target, np.float64)
    tgt = tgt / tgt.sum()
    for it in range(iters):
        freq = np.bincount(np.argmax(zr + b, axis=1), minlength=n_route) / n
        step = lr * scale * (np.log(tgt + 1e-4) - np.log(freq + 1e-4))
        b += step * (0.98 ** it)
    out = np.zeros(ncls, np.float32)
    out[:n_route] = b.astype(np.float32)
    return out


def calibrate_workload(wl, n_cal: int = 128, targets: Optional[Dict[int, np.ndarray]] = None, cal_seed_offset: int = 1 << 20,
                       threads: int = 0, progress=None) -> Dict[int, np.ndarray]:
    """Head-bias offsets for every routing expert of wl, from oracle logits on n_cal calibration images (request ids
    offset so they never coincide with workload requests).  targets[e]: routed-class distribution (default uniform).
    Fills wl.head_bias in place and returns it.  progress(e), if given, is called after every calibrated expert."""
    ids = np.arange(cal_seed_offset, cal_seed_offset + n_cal)
    x = wl.inputs(ids)
    for e in range(wl.graph.n_experts):
        k = int(wl.graph.succ_off[e + 1] - wl.graph.succ_off[e])
        if k <= 1:
            continue
        a = wl.archs[wl.expert_arch[e]]
        zero = np.zeros(a.n_classes, np.float32)
        wl.head_bias[e] = zero
        blob = wl.blob(e)
        z = np.stack([O.forward(a, blob, x[i]) for i in range(n_cal)]) if threads == 1 else _forward_many(a, blob, x, threads)
        tgt = np.full(k, 1.0 / k) if not targets or e not in targets else targets[e]
        wl.head_bias[e] = calibrate_bias(z, k, tgt)
        if progress:
            progress(e)
    return wl.head_bias


def _forward_many(arch, blob, x, threads):
    """All calibration images through one expert, in parallel, via the chain runner on a one-expert graph."""
    so = np.zeros(2, np.int32)
    r = O.run_chain([arch], [0], [blob], so, np.zeros(1, np.int32), x, None, 1, arch.n_classes, threads)
    return r["logits"]
