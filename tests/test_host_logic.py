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


@pytest.mark.parametrize("seed", range(4))
def test_two_level_policy_matches_oracle_random(B, oracle, seed):
    """The host tier's arrangement (Section 5.1: CPU memory as a cache in front of the SSD): the library's policy, once per
    level with the lower level asked once per device switch, against the oracle's two-level replay."""
    rng = np.random.default_rng(200 + seed)
    wl = W.config4(8, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    nbytes = [10] * E
    rule = seed % 3
    sim = oracle.TieredCacheSim(nbytes, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_device=5, cap_host=9 + seed, rule=rule,
                                in_use=seed % 2)
    dev = B.Policy(nbytes, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, 5, 0, eviction=rule, in_use_depth=seed % 2)
    host = B.Policy(nbytes, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, 9 + seed, 0, eviction=rule)

    def serve(e):
        need = np.zeros(E, np.uint8); need[e] = 1
        return host.stage(need)[1]

    reads = [(e, []) for e in host.init_fill()]
    loaded = dev.init_fill()
    for e in loaded:
        reads += serve(e)
    assert (loaded, reads) == sim.init_fill()
    for _ in range(40):
        hg = (rng.random(E) < rng.choice([0.1, 0.3, 0.5])).astype(np.uint8)
        order, sw = dev.stage(hg)
        reads = []
        for e, _ in sw:
            reads += serve(e)
        assert (order, sw, reads) == sim.stage(hg)


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


def test_profiler_arithmetic(B):
    """Latency model fit, maximum batch and arranging thresholds (paper Sections 4.2, 4.5) behind the C ABI: hand-made
    numbers, then random cases against the oracle's twin."""
    from oracle import profiler_oracle as PO
    K, Bc = B.coe_profiler_fit_latency([1, 2, 4, 8, 16], [103.0, 106.0, 112.0, 124.0, 148.0])     # exactly 3 n + 100
    assert abs(K - 3.0) < 1e-9 and abs(Bc - 100.0) < 1e-9
    K, Bc = B.coe_profiler_fit_latency([10, 20, 30], [25.0, 45.0, 59.0])                          # textbook least squares: 1.7 n + 9
    assert abs(K - 1.7) < 1e-9 and abs(Bc - 9.0) < 1e-9
    with pytest.raises(B.CoEError):
        B.coe_profiler_fit_latency([4, 4, 4], [1.0, 2.0, 3.0])
    # per-request latency 110, 60, 35, 22.5, 21.2, 21.0: within 5 % of the best from n = 16 on
    assert B.coe_profiler_max_batch([1, 2, 4, 8, 16, 32], [110, 120, 140, 180, 339.2, 672], 0.05) == 16
    assert B.coe_profiler_max_batch([1, 2, 4], [10, 20, 40]) == 1
    # K = 10, B = 1000, load = 800; half of the time useful: n >= 100 resident, 180 missing; a fifth: 25 and 45
    assert B.coe_profiler_arranging_window(10.0, 1000.0, 800.0, 0.5) == (100, 180)
    assert B.coe_profiler_arranging_window(10.0, 1000.0, 800.0, 0.2) == (25, 45)
    assert B.coe_profiler_arranging_window(10.0, 1000.0, 800.0, 0.0) == (0, 0)
    rng = np.random.default_rng(3)
    for _ in range(100):
        n = int(rng.integers(2, 9))
        ns = np.sort(rng.choice(np.arange(1, 600), size=n, replace=False))
        ts = rng.uniform(2, 20) * ns + rng.uniform(0, 2000) + rng.normal(0, 5, n)
        ts = np.maximum(ts, 1.0)
        k, b = B.coe_profiler_fit_latency(ns, ts)
        k2, b2 = PO.line_through(ns.tolist(), ts.tolist())
        assert abs(k - k2) <= 1e-9 * max(1, abs(k2)) and abs(b - b2) <= 1e-7 * max(1, abs(b2))
        tol = float(rng.choice([0.0, 0.05, 0.3]))
        assert B.coe_profiler_max_batch(ns, ts, tol) == PO.max_batch(ns.tolist(), ts.tolist(), tol)
        kk, bb, ld, eff = rng.uniform(1, 30), rng.uniform(0, 3000), rng.uniform(0, 2000), float(rng.choice([0.1, 0.2, 0.5, 0.8]))
        assert B.coe_profiler_arranging_window(kk, bb, ld, eff) == PO.arranging_thresholds(kk, bb, ld, eff)


def _run_window_search(B, total, curve, initial, margin, fit_points=2):
    ts, loaded = [], []
    st = B.coe_profiler_window_step(total, initial, margin, fit_points, ts)
    while st.status == B.COE_WINDOW_MEASURE:
        loaded.append(st.n_next)
        ts.append(curve(st.n_next))
        st = B.coe_profiler_window_step(total, initial, margin, fit_points, ts)
    return st, loaded, ts


def test_decay_window_search_reproduces_the_printed_case(B):
    """Section 5.4 prints one run of the search of Section 4.4: initial window size 15, error margin 5 %, final window
    "loading 28 to 39 experts" with a linear error of 7.7 % (Task A, 352 experts).  Eq. 1 gives the decay factor 0.85, so the
    window sizes are 15, 12.75, 10.8375 and the upper bounds 15, 27.75, 38.5875: the third window is 27.75..38.5875 = experts
    28 to 39, reached when the third throughput falls 7.7 % short of the line through the first two.  Oracle twin and
    library both have to land there."""
    from oracle import profiler_oracle as PO
    gold = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "section_5_4_memory_window.txt")):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=")
            gold[k.strip()] = float(v)
    w0, margin, total = gold["initial_window"], gold["error_margin"], int(gold["n_experts"])
    lo, hi, lin = int(gold["final_window_low_experts"]), int(gold["final_window_high_experts"]), gold["linear_error"]
    assert (w0, margin, total, lo, hi, lin) == (15, 0.05, 352, 28, 39, 0.077)
    assert [round(v, 4) for k in range(3) for v in PO.window_bounds(w0, k)] == [0, 15, 15, 27.75, 27.75, 38.5875]
    # throughputs 20 and 24 at 15 and 28 experts: the line predicts 28 at the third point; 7.7 % short of that is 25.844
    curve = {15: 20.0, 28: 24.0, 39: 28.0 * (1 - lin)}
    ref = PO.decay_window_search(total, lambda n: curve[n], w0, margin)
    assert ref["loaded"] == [15, lo, hi] and ref["experts"] == (lo, hi) and ref["stopped_by"] == "shortfall"
    assert abs(ref["linear_error"] - lin) < 1e-12
    st, loaded, ts = _run_window_search(B, total, lambda n: curve[n], w0, margin)
    assert loaded == [15, lo, hi] and (st.n_low, st.n_high) == (lo, hi) and st.status == B.COE_WINDOW_SHORTFALL
    assert abs(st.window_low - 27.75) < 1e-9 and abs(st.window_high - 38.5875) < 1e-9 and abs(st.linear_error - lin) < 1e-9
    # a shortfall inside the margin (4 %) does not stop the slide: the fourth window is 38.5875..47.799 = experts 39 to 48
    curve = {15: 20.0, 28: 24.0, 39: 28.0 * 0.96, 48: 10.0}
    st, loaded, ts = _run_window_search(B, 352, lambda n: curve[n], 15.0, 0.05)
    assert loaded == [15, 28, 39, 48] and (st.n_low, st.n_high) == (39, 48)
    assert PO.decay_window_search(352, lambda n: curve[n], 15.0, 0.05)["experts"] == (39, 48)


def test_decay_window_search_matches_the_oracle_twin(B):
    """Random throughput curves (rise, then fall somewhere), several initial windows, margins and expert counts: library and
    oracle twin measure at the same expert counts, stop at the same window for the same reason.  A curve that keeps rising
    ends when a window has loaded every expert (window sizes sum to 100, so totals below 100 are always reached)."""
    from oracle import profiler_oracle as PO
    rng = np.random.default_rng(5)
    for _ in range(200):
        total = int(rng.integers(3, 99))
        initial = float(rng.choice([5.0, 10.0, 15.0, 20.0, 30.0, 50.0]))
        margin = float(rng.choice([0.0, 0.05, 0.1, 0.3]))
        fit_points = int(rng.integers(2, 5))
        peak = rng.uniform(0, 1.5) * total
        noise = rng.normal(0, 0.02, total + 1)
        curve = lambda n: 100.0 + 10.0 * min(n, peak) - 25.0 * max(0.0, n - peak) + noise[n]
        ref = PO.decay_window_search(total, curve, initial, margin, fit_points)
        st, loaded, ts = _run_window_search(B, total, curve, initial, margin, fit_points)
        assert loaded == ref["loaded"], (total, initial, margin, fit_points)
        assert (st.n_low, st.n_high) == ref["experts"]
        assert ("shortfall" if st.status == B.COE_WINDOW_SHORTFALL else "end") == ref["stopped_by"]
        assert abs(st.linear_error - ref["linear_error"]) < 1e-9
        assert abs(st.window_low - ref["window"][0]) < 1e-9 and abs(st.window_high - ref["window"][1]) < 1e-9
    with pytest.raises(B.CoEError):
        B.coe_profiler_window_step(10, 0.0, 0.05, 2, [])
    with pytest.raises(B.CoEError):
        B.coe_profiler_window_step(10, 15.0, 0.05, 1, [])


def test_assigning_rule_matches_oracle(B):
    """The library's executor assignment (least work so far, lowest number among equals) against the oracle's, which
    evaluates the paper's two criteria (smallest total over all queues, then smallest own queue) literally."""
    from oracle.arrange import assign
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(0, 40)); k = int(rng.integers(1, 5))
        cost = rng.integers(0, 50, n) if rng.random() < 0.5 else rng.integers(1, 4, n) * 1000
        assert B.coe_assign_executors(cost, k).tolist() == assign(cost.tolist(), k)


def test_memory_scores_and_expert_budget(B):
    """Section 4.5: footprints normalised to memory scores; Section 4.4: with inference at the maximum batch, experts get the
    rest of the memory.  Library against the oracle's twin and against hand values."""
    from oracle import profiler_oracle as PO
    nbytes = [46_900_000, 22_300_000, 171_400_000, 22_300_000]          # ResNet-50-, ResNet-18-, ViT-B/16-shaped blobs
    score, unit = B.coe_profiler_memory_scores(nbytes)
    want, wunit = PO.memory_scores(nbytes)
    assert unit == wunit == 22_300_000 and np.allclose(score, want, rtol=0, atol=1e-12)
    assert score[1] == score[3] == 1.0 and abs(score[2] - 7.686098654708520) < 1e-12
    # 12 GB of device memory (the paper's RTX 3080Ti), 1 GB reserved, 9.5 MB of activations per request, maximum batch 64
    left, scores = B.coe_profiler_expert_budget(12 * 10**9, 10**9, 9_500_000, 64, unit)
    assert left == PO.expert_budget(12 * 10**9, 10**9, 9_500_000, 64) == 10_392_000_000
    assert abs(scores - left / unit) < 1e-9
    assert B.coe_profiler_expert_budget(10**9, 0, 10**9, 4096, unit) == (0, 0.0)        # the batch alone exceeds the memory
    for bad in ([], [5, 0], [-1]):
        with pytest.raises(B.CoEError):
            B.coe_profiler_memory_scores(bad)
    with pytest.raises(B.CoEError):
        B.coe_profiler_expert_budget(10, 0, 1, 1, 0)


def test_executable_batch_is_the_smaller_of_memory_and_profile(B):
    """Section 4.2 "Request splitting": hand values, the oracle's twin, and the consistency with the expert budget: what is
    left after the experts' share holds exactly the batch the budget was computed for."""
    from oracle import profiler_oracle as PO
    assert B.coe_profiler_executable_batch(10**9, 9_500_000, 512) == PO.executable_batch(10**9, 9_500_000, 512) == 105
    assert B.coe_profiler_executable_batch(10**10, 9_500_000, 512) == 512
    assert B.coe_profiler_executable_batch(9_499_999, 9_500_000, 512) == 0
    total, reserve, per_req, mb = 12 * 10**9, 10**9, 9_500_000, 64
    experts, _ = B.coe_profiler_expert_budget(total, reserve, per_req, mb, 1)
    assert B.coe_profiler_executable_batch(total - reserve - experts, per_req, 10**6) == mb
    with pytest.raises(B.CoEError):
        B.coe_profiler_executable_batch(1, 0, 1)


def test_usage_probabilities_from_sample_paths(B, oracle):
    """Section 4.5 "Expert information": probabilities recorded from a sample run.  Hand case, the oracle's twin on random
    paths through a DAG, and the closed form of a workload whose routes are drawn with known probabilities."""
    from oracle import profiler_oracle as PO
    paths = np.array([[0, 2, -1], [0, 3, 5], [1, 3, 5], [0, 2, -1]], np.int32)
    got = B.coe_profiler_usage_probabilities(paths, 6)
    assert got.tolist() == [0.75, 0.25, 0.5, 0.5, 0.0, 0.5] == PO.usage_probabilities(paths, 6)
    rng = np.random.default_rng(4)
    wl = W.config4(2000, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    rnd = np.full((2000, 3), -1, np.int32)
    for r in range(2000):
        e = int(wl.first_expert[r])
        for s_ in range(3):
            rnd[r, s_] = e
            succ = wl.graph.successors(e)
            if len(succ) == 0:
                break
            e = int(succ[rng.integers(len(succ))])
            if e < 0:
                break
    got = B.coe_profiler_usage_probabilities(rnd, E)
    assert np.allclose(got, PO.usage_probabilities(rnd, E), rtol=0, atol=1e-7)
    assert abs(got[:4].sum() - 1.0) < 1e-6                                  # every request starts at one first-tier expert
    assert np.abs(got - np.asarray(wl.usage_prob)).max() < 0.05            # uniform random routes: the workload's own probabilities
    for bad in (np.array([[7]], np.int32), np.array([[-2]], np.int32)):
        with pytest.raises(B.CoEError):
            B.coe_profiler_usage_probabilities(bad, 6)
