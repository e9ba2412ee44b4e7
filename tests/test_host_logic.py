"""Host-side logic of the library that needs no GPU: exported symbols, graph validation, cache policy vs the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import coe_workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2503_02354_amd import build
    if build.needs_build():
        build.build()
    from paper_2503_02354_amd import binding
    return binding


def test_library_exports_every_declared_symbol(B):
    hdr = open(os.path.join(ROOT, "include", "coe.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(coe_[a-z_0-9]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    L = C.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(L, name), name


def test_validate_graph(B):
    g = W.tree_graph(4)
    assert B.coe_validate_graph(4, g.succ_off, g.succ, [3, 1, 1, 1]) == B.COE_OK
    assert B.coe_validate_graph(4, g.succ_off, g.succ, [2, 1, 1, 1]) == B.COE_EGRAPH        # more routes than classes
    bad = W.graph_from_lists([[1], [2], [0]])                                                # cycle
    assert B.coe_validate_graph(3, bad.succ_off, bad.succ) == B.COE_EGRAPH
    self_loop = W.graph_from_lists([[0]])
    assert B.coe_validate_graph(1, self_loop.succ_off, self_loop.succ) == B.COE_EGRAPH
    oob = W.graph_from_lists([[1, 5], []])
    assert B.coe_validate_graph(2, oob.succ_off, oob.succ) == B.COE_EGRAPH
    final = W.graph_from_lists([[1, -1], [-1]])
    assert B.coe_validate_graph(2, final.succ_off, final.succ) == B.COE_OK
    dag = W.config4(8, hw=32, tiers=(3, 5, 7), width=8, fan=(3, 2), calibrated=False).graph    # shared downstream experts
    assert B.coe_validate_graph(dag.n_experts, dag.succ_off, dag.succ) == B.COE_OK
    assert B.coe_validate_graph(0, g.succ_off, g.succ) == B.COE_EINVAL


def test_create_without_gpu_fails_loudly(B):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.CoEError) as ei:
        B.Context(max_requests=4)
    assert ei.value.code == B.COE_EDEVICE


def _compare_policy(B, oracle, nbytes, prob, graph, cap_experts, cap_bytes, stages, rule=0, depth=0):
    sim = oracle.CacheSim(nbytes, prob, graph.succ_off, graph.succ, cap_experts, cap_bytes, rule=rule, in_use=depth)
    pol = B.Policy(nbytes, prob, graph.succ_off, graph.succ, cap_experts, cap_bytes, eviction=rule, in_use_depth=depth)
    assert sim.init_fill() == pol.init_fill()
    for hg in stages:
        try:
            want = sim.stage(hg)
        except MemoryError:
            with pytest.raises(MemoryError):
                pol.stage(hg)
            return
        got = pol.stage(hg)
        assert got == want
        assert np.array_equal(sim.resident(), pol.resident())


def test_policy_matches_oracle_on_hand_cases(B, oracle):
    g = W.graph_from_lists([[2, 3], [4], [], [], [], []])
    _compare_policy(B, oracle, [50, 10, 20, 40, 30, 60], [0.0, 0.0, 0.9, 0.8, 0.7, 0.6], g, 0, 150,
                    [[0, 1, 0, 0, 0, 0], [1, 0, 0, 0, 0, 0]])
    g = W.graph_from_lists([[1], [2], [], [], []])
    _compare_policy(B, oracle, [100, 10, 50, 10, 30], [0.0, 0.9, 0.8, 0.1, 0.05], g, 0, 70, [[0, 0, 0, 0, 1]])
    g = W.tree_graph(4)
    _compare_policy(B, oracle, [10] * 4, [1.0, 0.5, 0.3, 0.2], g, 2, 0, [[0, 1, 1, 1], [1, 0, 0, 0], [0, 1, 0, 1]])


@pytest.mark.parametrize("seed", range(6))
def test_policy_matches_oracle_random(B, oracle, seed):
    rng = np.random.default_rng(seed)
    wl = W.config4(8, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    nbytes = rng.integers(5, 30, E) if seed % 2 else np.full(E, 10)
    prob = np.round(np.asarray(wl.usage_prob), 2) if seed % 3 == 0 else wl.usage_prob      # rounded: exercises ties
    stages = [(rng.random(E) < rng.choice([0.1, 0.3, 0.6])).astype(np.uint8) for _ in range(40)]
    _compare_policy(B, oracle, nbytes, prob, wl.graph, 0 if seed % 2 else 6, 110 if seed % 2 else 0, stages)


@pytest.mark.parametrize("rule", [1, 2])
@pytest.mark.parametrize("seed", range(4))
def test_comparison_rules_match_oracle_random(B, oracle, seed, rule):
    """Least-recently-used and first-in-first-out replacement (the rules of the paper's comparison systems,
    Section 5.1): the library's policy against the oracle's replay, random stages, count and byte caps."""
    rng = np.random.default_rng(50 + seed)
    wl = W.config4(8, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    nbytes = rng.integers(5, 30, E) if seed % 2 else np.full(E, 10)
    stages = [(rng.random(E) < rng.choice([0.1, 0.3, 0.6])).astype(np.uint8) for _ in range(40)]
    _compare_policy(B, oracle, nbytes, wl.usage_prob, wl.graph, 0 if seed % 2 else 6, 110 if seed % 2 else 0, stages, rule=rule,
                    depth=seed % 3)


@pytest.mark.parametrize("depth", [1, 2, 3])
@pytest.mark.parametrize("seed", range(4))
def test_in_use_depth_matches_oracle_random(B, oracle, seed, depth):
    """Two-stage rule with the experts of the preceding groups protected while a load is in flight."""
    rng = np.random.default_rng(80 + seed)
    wl = W.config4(8, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    nbytes = rng.integers(5, 30, E) if seed % 2 else np.full(E, 10)
    stages = [(rng.random(E) < rng.choice([0.1, 0.3, 0.6])).astype(np.uint8) for _ in range(40)]
    _compare_policy(B, oracle, nbytes, wl.usage_prob, wl.graph, 0 if seed % 2 else 8, 130 if seed % 2 else 0, stages, depth=depth)


def test_policy_zipf_tree_keeps_hot_experts(B, oracle):
    # config-3 structure at small scale: root + Zipf leaves, cap 5: after many stages the hottest leaves stay resident
    wl = W.config3(64, hw=32, n_experts=12, width=8, cap=5, arrival_batch=16, calibrated=False)
    E = 12
    nbytes = [100] * E
    rng = np.random.default_rng(0)
    p = np.asarray(wl.usage_prob[1:])
    stages = []
    for _ in range(30):
        hg = np.zeros(E, np.uint8); hg[0] = 1
        leaves = rng.choice(np.arange(1, E), size=6, p=p / p.sum())
        hg[leaves] = 1
        stages.append(hg)
    _compare_policy(B, oracle, nbytes, wl.usage_prob, wl.graph, 5, 0, stages)


def test_arranging_rule_matches_oracle(B):
    """The library's arranging-window rule (host only) against the oracle's, on random queues."""
    from oracle.arrange import stays_queued
    rng = np.random.default_rng(7)
    for _ in range(200):
        E = int(rng.integers(1, 40))
        count = rng.integers(0, 12, E); age = rng.integers(0, 6, E); res = rng.integers(0, 2, E)
        mr = rng.integers(0, 10, E); mm = rng.integers(0, 10, E); mw = rng.integers(0, 6, E)
        got = B.coe_arrange_defer(count, age, res, mr, mm, mw)
        want = [stays_queued(int(count[e]), int(age[e]), bool(res[e]), int(mr[e]), int(mm[e]), int(mw[e])) for e in range(E)]
        assert got.tolist() == want


def test_profiler_arithmetic():
    """Latency model fit, batch plateau and arranging thresholds (paper Sections 4.2, 4.5) on hand-made numbers."""
    from paper_2503_02354_amd import profiler as P
    K, Bc = P.fit_latency([1, 2, 4, 8, 16], [103.0, 106.0, 112.0, 124.0, 148.0])     # exactly 3 n + 100
    assert abs(K - 3.0) < 1e-9 and abs(Bc - 100.0) < 1e-9
    K, Bc = P.fit_latency([10, 20, 30], [25.0, 45.0, 59.0])                           # textbook least squares: 1.7 n + 9
    assert abs(K - 1.7) < 1e-9 and abs(Bc - 9.0) < 1e-9
    # per-request latency 110, 60, 35, 22.5, 21.2, 21.0: within 5 % of the best from n = 16 on
    assert P.plateau_batch([1, 2, 4, 8, 16, 32], [110, 120, 140, 180, 339.2, 672], tol=0.05) == 16
    assert P.plateau_batch([1, 2, 4], [10, 20, 40]) == 1
    # K = 10, B = 1000, load = 800; half of the time useful: n >= 100 resident, 180 missing; a fifth: 25 and 45
    assert P.arranging_window(10.0, 1000.0, 800.0, 0.5, 8) == (100, 180, 8)
    assert P.arranging_window(10.0, 1000.0, 800.0, 0.2, 3) == (25, 45, 3)
    assert P.arranging_window(10.0, 1000.0, 800.0, 0.0, 3) == (0, 0, 3)


def test_decay_window_search_hand_worked():
    """Section 4.4 on hand-made numbers.  20 experts of equal usage: each covers 5 % of the usage.  Initial window 20 %,
    decay factor 0.8: upper bounds 20, 36, 48.8, 59.04, 67.23, ... % -> 4, 8, 10, 12, 14 experts.  Throughput rises by 10
    per window (100, 110, 120, 130) and then falls to 90 at 14 experts: the line through the first four values
    predicts 140, the shortfall (140 - 90) / 140 = 0.36 exceeds the margin, the search stops in the window 59.04..67.23 %
    and its middle (63.1 %) is covered by 13 experts."""
    from paper_2503_02354_amd import profiler as P
    usage = [1.0] * 20
    assert [P.experts_for_usage(usage, q) for q in (5, 5.1, 20, 36, 48.8, 59.04, 100)] == [1, 2, 4, 8, 10, 12, 20]
    curve = {4: 100.0, 8: 110.0, 10: 120.0, 12: 130.0, 14: 90.0}
    seen = []
    out = P.decay_window_search(usage, lambda n: (seen.append(n), curve[n])[1], initial_window=20.0, min_points=3,
                                error_margin=0.1, pick=0.5)
    assert seen == [4, 8, 10, 12, 14]
    assert out["stopped_by"] == "shortfall" and out["n_experts"] == 13
    assert abs(out["window"][0] - 59.04) < 1e-9 and abs(out["window"][1] - 67.232) < 1e-9
    # a throughput that keeps following the line: the windows (30 %, then x 0.7 each: upper bounds 30, 51, 65.7, 75.99,
    # 83.19, 88.24, 91.76 %) shrink until the next one (94.24 %) adds no expert to the 19 that cover 91.76 %
    out = P.decay_window_search(usage, lambda n: 100.0 + 2.0 * n, initial_window=30.0, pick=1.0)
    assert out["stopped_by"] == "end" and abs(out["window"][1] - 91.76457) < 1e-6 and out["n_experts"] == 19
    assert [v[1] for v in out["trace"]] == [6, 11, 14, 16, 17, 18, 19]
    # a skewed CDF: Zipf(1.1) over 63 leaves reaches 74.9 % of the usage with its 15 most used experts
    z = W.zipf_probs(63, 1.1)
    assert P.experts_for_usage(z, 74.0) == 15 and P.experts_for_usage(z, 25.0) == 1


def test_assigning_rule_matches_oracle(B):
    """The library's executor assignment (least work so far, lowest number among equals) against the oracle's, which
    evaluates the paper's two criteria (smallest total over all queues, then smallest own queue) literally."""
    from oracle.arrange import assign
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(0, 40)); k = int(rng.integers(1, 5))
        cost = rng.integers(0, 50, n) if rng.random() < 0.5 else rng.integers(1, 4, n) * 1000
        assert B.coe_assign_executors(cost, k).tolist() == assign(cost.tolist(), k)
