"""Pins for the oracle's integer parts: request arranging (regroup), splitting, the routed chain and the cache policy."""
import itertools

import numpy as np
import pytest

import coe_workloads as W


# ---------------------------------------------------------------------------------------------
# regroup (request arranging) and splitting
# ---------------------------------------------------------------------------------------------
def test_regroup_exhaustive_tiny(oracle):
    # the answer is unique (grouped by expert, arrival order kept inside a group), so brute force pins it
    for n in range(0, 7):
        for E in (1, 2, 3):
            for cur in itertools.product(range(-1, E), repeat=n):
                r = oracle.regroup(np.array(cur, np.int32), E)
                want = sorted([i for i in range(n) if cur[i] >= 0], key=lambda i: (cur[i], i))
                assert r["perm"].tolist() == want
                assert r["cnt"].tolist() == [sum(1 for c in cur if c == e) for e in range(E)]
                assert r["off"].tolist() == [sum(1 for c in cur if 0 <= c < e) for e in range(E + 1)]
                for i in range(n):
                    assert r["inv"][i] == (want.index(i) if cur[i] >= 0 else -1)


def test_regroup_invariants_large(oracle):
    rng = np.random.default_rng(0)
    n, E = 5000, 37
    cur = rng.integers(-1, E, n).astype(np.int32)
    r = oracle.regroup(cur, E)
    perm = r["perm"]
    assert sorted(perm.tolist()) == np.nonzero(cur >= 0)[0].tolist()            # a permutation of the pending set
    keys = cur[perm]
    assert np.all(np.diff(keys) >= 0)                                           # grouped by expert
    same = np.diff(keys) == 0
    assert np.all(np.diff(perm)[same] > 0)                                      # arrival order kept inside a group
    assert r["cnt"].sum() == r["n_pending"] == len(perm) and r["off"][-1] == len(perm)
    assert np.array_equal(r["off"][1:] - r["off"][:-1], r["cnt"])
    assert np.array_equal(r["inv"][perm], np.arange(len(perm)))


def test_split_covers_groups(oracle):
    off = np.array([0, 5, 5, 12, 13], np.int32)
    ch = oracle.split(off, [2, 0, 3, 1], 4)
    # by hand: 7 requests, at most 4 per batch -> 2 batches of ceil(7/2) = 4 and the rest; 5 requests -> 2 batches of 3 and 2
    assert ch.tolist() == [[2, 5, 4], [2, 9, 3], [0, 0, 3], [0, 3, 2], [3, 12, 1]]
    # fewest batches, as even as consecutive cutting allows: 9 -> 3+3+3 (not 4+4+1), 10 -> 4+4+2, 8 -> 4+4, 4 -> 4, 1 -> 1
    off2 = np.array([0, 9, 19, 27, 31, 32], np.int32)
    assert oracle.split(off2, [0, 1, 2, 3, 4], 4)[:, 2].tolist() == [3, 3, 3, 4, 4, 2, 4, 4, 4, 1]
    rng = np.random.default_rng(1)
    cnt = rng.integers(0, 40, 20); off = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
    for mb in (1, 7, 64):
        ch = oracle.split(off, list(range(20)), mb)
        assert ch[:, 2].max() <= mb and ch[:, 2].min() >= 1
        covered = np.concatenate([np.arange(s, s + c) for _, s, c in ch])
        assert np.array_equal(covered, np.arange(off[-1]))
        for e, s, c in ch:
            assert off[e] <= s and s + c <= off[e + 1]
        assert len(ch) == sum(-(-int(c) // mb) for c in cnt)


# ---------------------------------------------------------------------------------------------
# routed chain with planted weights
# ---------------------------------------------------------------------------------------------
def _head_only_arch(ncls, c=3, hw=2):
    layers = np.array([[W.OP_HEAD, 0, -1, -1, ncls, 0, 0, 0, 0, 0, 0, 0]], np.int32)
    return W.Arch("head_only", W.DT_F32, hw, hw, c, ncls, layers, [1.0])


def _planted_blob(arch, w, b):
    specs, nbytes = W.blob_layout(arch)
    blob = np.zeros(nbytes, np.uint8)
    blob[specs[0].offset:specs[0].offset + specs[0].nbytes] = np.asarray(w, np.float32).reshape(-1).view(np.uint8)
    blob[specs[1].offset:specs[1].offset + specs[1].nbytes] = np.asarray(b, np.float32).reshape(-1).view(np.uint8)
    return blob


def test_chain_planted_routes(oracle):
    # experts see only the per-channel mean m = (m0, m1, m2).  Expert 0 routes over its first 3 classes:
    #   class 0 -> expert 1, class 1 -> expert 2, class 2 -> final (-1);  class 3 is never a route even if largest.
    a = _head_only_arch(4)
    e0 = _planted_blob(a, [[1, 0, 0], [0, 1, 0], [0, 0, 1], [5, 5, 5]], [0, 0, 0, 100])
    e1 = _planted_blob(a, [[2, 0, 0], [0, 0, 0], [0, 0, 0], [0, 0, 0]], [0, 1, 2, 3])     # leaf: logits (2 m0, 1, 2, 3)
    e2 = _planted_blob(a, [[0, 0, 0], [0, 0, 0], [0, 0, 0], [0, -1, 0]], [7, 7, 7, 0])    # routes: class 0 -> expert 1
    g = W.graph_from_lists([[1, 2, -1], [], [1, 1, 1]])
    means = np.array([[3, 1, 2], [1, 3, 2], [1, 2, 3], [2, 2, 1], [0, 0, 0]], np.float32)
    x = np.broadcast_to(means[:, None, None, :], (5, 2, 2, 3)).astype(np.float32).copy()
    x[:, 0, 0, :] += 1; x[:, 1, 1, :] -= 1                                          # same mean, not constant
    r = oracle.run_chain([a], [0, 0, 0], [e0, e1, e2], g.succ_off, g.succ, x, None, 3, 4)
    assert r["path"].tolist() == [[0, 1, -1], [0, 2, 1], [0, -1, -1], [0, 1, -1], [0, 1, -1]]
    np.testing.assert_allclose(r["logits"][0], [6, 1, 2, 3])      # expert 1 on mean (3,1,2)
    np.testing.assert_allclose(r["logits"][1], [2, 1, 2, 3])      # via expert 2 then expert 1 on mean (1,3,2)
    np.testing.assert_allclose(r["logits"][2], [1, 2, 3, 130])    # final at expert 0: its own logits
    # ties take the lowest class: request 3 (2,2,1) -> class 0; request 4 (0,0,0) -> class 0
    # first_expert overrides the start
    r2 = oracle.run_chain([a], [0, 0, 0], [e0, e1, e2], g.succ_off, g.succ, x, np.array([2, 1, 0, 2, 1], np.int32), 3, 4)
    assert r2["path"].tolist() == [[2, 1, -1], [1, -1, -1], [0, -1, -1], [2, 1, -1], [1, -1, -1]]


def _valid_paths(path, graph, first):
    for r, p in enumerate(path):
        p = [int(v) for v in p if v >= 0]
        assert p[0] == (0 if first is None else int(first[r]))
        for a, b in zip(p, p[1:]):
            assert b in graph.successors(a).tolist()
        last = p[-1]
        assert len(graph.successors(last)) == 0 or -1 in graph.successors(last).tolist() or len(p) == path.shape[1]


def test_chain_paths_valid_and_schedule_independent(oracle):
    wl = W.config4(48, hw=32, tiers=(3, 5, 7), width=8, fan=(3, 2), calibrated=False)
    blobs = [wl.blob(e) for e in range(wl.graph.n_experts)]
    x = wl.inputs(range(48))
    r = oracle.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, x, wl.first_expert, 3, wl.max_classes)
    _valid_paths(r["path"], wl.graph, wl.first_expert)
    assert np.all(r["path"][:, 2] >= 0)                      # three-stage DAG: every request reaches stage 3
    # results do not depend on which other requests are present, nor on their order
    idx = np.array([40, 3, 17, 5])
    r2 = oracle.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, x[idx], wl.first_expert[idx], 3,
                          wl.max_classes, threads=1)
    assert np.array_equal(r2["path"], r["path"][idx]) and np.array_equal(r2["logits"], r["logits"][idx])


def test_chain_equals_stagewise_grouped_execution(oracle):
    # grouping requests by expert, running groups in any order and regrouping between stages gives the same result
    wl = W.config2(40, hw=32, n_experts=5, width=8, calibrated=False)
    wl.head_bias[0] = np.zeros(16, np.float32)
    blobs = [wl.blob(e) for e in range(5)]
    x = wl.inputs(range(40))
    ref = oracle.run_chain(wl.archs, wl.expert_arch, blobs, wl.graph.succ_off, wl.graph.succ, x, None, 2, 16)
    cur = np.zeros(40, np.int32); logits = np.zeros((40, 16), np.float32); path = np.full((40, 2), -1, np.int32)
    rng = np.random.default_rng(5)
    for stage in range(2):
        rg = oracle.regroup(cur, 5)
        order = [e for e in rng.permutation(5) if rg["cnt"][e] > 0]
        nxt = np.full(40, -1, np.int32)
        for e, s, c in oracle.split(rg["off"], order, 7):
            for r_ in rg["perm"][s:s + c]:
                lg = oracle.forward(wl.archs[0], blobs[e], x[r_])
                logits[r_] = lg; path[r_, stage] = e
                succ = wl.graph.successors(e)
                if len(succ):
                    nxt[r_] = succ[int(np.argmax(lg[:len(succ)]))]
        cur = nxt
    assert np.array_equal(path, ref["path"]) and np.array_equal(logits, ref["logits"])


# ---------------------------------------------------------------------------------------------
# cache policy: hand-made pools
# ---------------------------------------------------------------------------------------------
def test_cache_init_fill_descending_probability(oracle):
    g = W.tree_graph(6)
    sim = oracle.CacheSim([10] * 6, [1.0, 0.1, 0.4, 0.2, 0.4, 0.05], g.succ_off, g.succ, cap_experts=4)
    assert sim.init_fill() == [0, 2, 4, 3]                     # ties: lower id first; stops when full
    assert sim.resident().tolist() == [True, False, True, True, True, False]
    simb = oracle.CacheSim([10, 30, 10, 10, 10, 10], [1.0, 0.9, 0.4, 0.2, 0.4, 0.05], g.succ_off, g.succ, cap_bytes=35)
    assert simb.init_fill() == [0]                             # expert 1 (30 bytes) does not fit: filling stops there


def test_cache_stage2_ascending_probability(oracle):
    # root resident, so no leaf lacks its predecessor: only the usage-probability stage applies
    g = W.tree_graph(6)
    prob = [1.0, 0.30, 0.25, 0.20, 0.15, 0.10]
    sim = oracle.CacheSim([10] * 6, prob, g.succ_off, g.succ, cap_experts=3)
    assert sim.init_fill() == [0, 1, 2]
    order, sw = sim.stage([False, True, False, False, True, True])
    assert order == [1, 4, 5]                                  # resident group first, then misses by id
    # loading 4: candidates 0 (p=1.0) and 2 (p=.25); 1 still has its group to run when... it ran first, so 1 is evictable:
    # lowest probability among {0, 1, 2} not waiting = 2 -> evict 2.  loading 5: among {0, 1, 4}: 4 has run -> p=.15 lowest
    assert sw == [(4, [2]), (5, [4])]
    assert sim.resident().tolist() == [True, True, False, False, False, True]


def test_cache_stage1_dependents_without_predecessor_first(oracle):
    # chain graph: 0 -> {2}, 1 -> {3}, 2 and 3 leaves, 4 independent root (no predecessor)
    g = W.graph_from_lists([[2], [3], [], [], []])
    nbytes = [10, 10, 30, 20, 10]
    prob = [0.5, 0.5, 0.9, 0.8, 0.01]
    sim = oracle.CacheSim(nbytes, prob, g.succ_off, g.succ, cap_bytes=70)
    # make the pool {2, 3, 4} + 0 by loading in probability order: 2 (30), 3 (20), then 0 (10) fits, 1 (10) fits = 70
    assert sim.init_fill() == [2, 3, 0, 1]
    # evict nothing yet; now request expert 4 (10 bytes): pool is full (70).  Stage 1 candidates: experts with predecessors,
    # none of which is resident or has a group: 2's predecessor 0 is resident, 3's predecessor 1 is resident -> none.
    # Stage 2: ascending probability among {0, 1, 2, 3}: 0 (0.5, lower id) -> evict 0.
    order, sw = sim.stage([False, False, False, False, True])
    assert sw == [(4, [0])]
    # request expert 0 again (10 bytes, pool {1, 2, 3, 4} at 70)
    order, sw = sim.stage([True, False, False, False, False])
    assert sw == [(0, [4])]
    # expert 0 is requested, so its dependent 2 counts as having a predecessor around -> protected; stage 2 evicts 4 (p=0.01)
    assert sim.resident().tolist() == [True, True, True, True, False]


def test_cache_stage1_order_descending_bytes(oracle):
    # predecessors 0 and 1 are neither resident nor requested; their dependents 2, 3, 4 are resident
    g = W.graph_from_lists([[2, 3], [4], [], [], [], []])
    nbytes = [50, 10, 20, 40, 30, 60]
    prob = [0.0, 0.0, 0.9, 0.8, 0.7, 0.6]
    sim = oracle.CacheSim(nbytes, prob, g.succ_off, g.succ, cap_bytes=150)
    assert sim.init_fill() == [2, 3, 4, 5]                     # 20+40+30+60 = 150
    # load expert 1 (10 bytes): stage 1 candidates {2, 3, 4} (5 has no predecessor) by descending bytes: 3 (40) -> fits, stop
    order, sw = sim.stage([False, True, False, False, False, False])
    assert sw == [(1, [3])]
    # load expert 0 (50 bytes): resident {1, 2, 4, 5} = 120.  Expert 0 itself is requested, so its dependent 2 is protected;
    # 4's predecessor 1 is resident -> protected; stage 1 empty.  Stage 2 ascending probability: 1 (0.0) frees 10 -> 110+50 > 150;
    # next 5 (0.6) frees 60 -> fits.
    order, sw = sim.stage([True, False, False, False, False, False])
    assert sw == [(0, [1, 5])]
    assert sim.resident().tolist() == [True, False, True, False, True, False]


def test_cache_stage1_candidates_fixed_at_the_miss(oracle):
    # chain 0 -> 1 -> 2 plus independent 3, 4.  Resident {1, 2, 3}; 0 absent.  The dependents-without-predecessor set is
    # taken when the miss occurs ("sorted ... and evicted sequentially"): evicting 1 does not add 2 to it.
    g = W.graph_from_lists([[1], [2], [], [], []])
    sim = oracle.CacheSim([100, 10, 50, 10, 30], [0.0, 0.9, 0.8, 0.1, 0.05], g.succ_off, g.succ, cap_bytes=70)
    assert sim.init_fill() == [1, 2, 3]
    order, sw = sim.stage([False, False, False, False, True])
    # stage 1: {1} (10 bytes) -> 60 + 30 > 70; stage 2 ascending probability: 3 (0.1) -> 50 + 30 > 70; 2 (0.8) -> fits
    assert sw == [(4, [1, 3, 2])]


def test_cache_never_evicts_waiting_group_and_reports_no_fit(oracle):
    g = W.tree_graph(4)
    sim = oracle.CacheSim([10] * 4, [1.0, 0.5, 0.3, 0.2], g.succ_off, g.succ, cap_experts=2)
    assert sim.init_fill() == [0, 1]
    order, sw = sim.stage([False, True, True, True])
    assert order == [1, 2, 3]
    assert sw == [(2, [1]), (3, [2])]                          # 1 ran already; root (p=1) kept; then 2 (ran) goes before root
    # capacity 1 and two residents impossible: an expert larger than the cap cannot fit
    sim2 = oracle.CacheSim([10, 100], [1.0, 0.5], W.tree_graph(2).succ_off, W.tree_graph(2).succ, cap_bytes=50)
    sim2.init_fill()
    with pytest.raises(MemoryError):
        sim2.stage([False, True])


def test_cache_invariants_random(oracle):
    rng = np.random.default_rng(3)
    wl = W.config4(16, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    nbytes = rng.integers(5, 30, E)
    cap = 120
    sim = oracle.CacheSim(nbytes, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_bytes=cap)
    sim.init_fill()
    for _ in range(30):
        hg = rng.random(E) < 0.2
        before = sim.resident()
        order, sw = sim.stage(hg)
        after = sim.resident()
        assert sorted(order) == np.nonzero(hg)[0].tolist()
        assert int(nbytes[after].sum()) <= cap
        if order:
            assert after[order[-1]]                                                 # the last group's expert is still there
        for e, victims in sw:
            assert e not in victims and len(set(victims)) == len(victims)
        assert [e for e, _ in sw] == [e for e in order if not before[e]]          # one load per missing group, no more
        n_hit = int(before[hg].sum())
        assert all(before[e] for e in order[:n_hit])                              # hits run first


def test_two_level_cache_hand_worked(oracle):
    """Root 0 -> leaves 1..5 with usage probabilities 1.0, .30, .25, .20, .15, .10; two experts fit the device, four the host
    level.  Worked by hand from the reading: the host level fills first ([0, 1, 2, 3]), serves the device's fill ([0, 1]) without
    a read, and afterwards every device switch is one request to it."""
    g = W.tree_graph(6)
    sim = oracle.TieredCacheSim([10] * 6, [1.0, 0.30, 0.25, 0.20, 0.15, 0.10], g.succ_off, g.succ, cap_device=2, cap_host=4)
    loaded, reads = sim.init_fill()
    assert loaded == [0, 1] and reads == [(0, []), (1, []), (2, []), (3, [])]
    # a group for leaf 4: the device evicts its least probable expert (1); the host level misses and evicts ITS least probable (3)
    order, sw, reads = sim.stage([False, False, False, False, True, False])
    assert order == [4] and sw == [(4, [1])] and reads == [(4, [3])]
    assert sim.host.resident().tolist() == [True, True, True, False, True, False]
    # groups for 3 and 5, both missing on the device.  Device: 3 replaces 4; 3 has run when 5 is loaded and is the least
    # probable again.  Host level: 3 is read back (4 leaves), then 5 replaces 3: each level thrashes its own coldest slot
    order, sw, reads = sim.stage([False, False, False, True, False, True])
    assert order == [3, 5] and sw == [(3, [4]), (5, [3])] and reads == [(3, [4]), (5, [3])]
    assert sim.dev.resident().tolist() == [True, False, False, False, False, True]
    assert sim.host.resident().tolist() == [True, True, True, False, False, True]
    # leaf 2 is on the host level: a device switch without a read
    order, sw, reads = sim.stage([False, False, True, False, False, False])
    assert sw == [(2, [5])] and reads == []


def test_two_level_cache_invariants_random(oracle):
    rng = np.random.default_rng(11)
    wl = W.config4(16, hw=32, tiers=(4, 8, 12), width=8, fan=(3, 2), calibrated=False)
    E = wl.graph.n_experts
    for cap_host in (8, 12, E):
        sim = oracle.TieredCacheSim([10] * E, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_device=5, cap_host=cap_host)
        loaded, reads = sim.init_fill()
        assert [e for e, _ in reads[:cap_host]] == sorted(range(E), key=lambda e: (-wl.usage_prob[e], e))[:cap_host]
        seen = {e for e, _ in reads}
        n_sw = n_rd = 0
        for _ in range(40):
            hg = rng.random(E) < 0.25
            on_host = sim.host.resident()
            order, sw, reads = sim.stage(hg)
            assert all(sim.host.resident()[e] for e, _ in sw[-1:])               # the newest load's source is still there
            assert [e for e, _ in reads] == [e for e in dict.fromkeys(e for e, _ in reads)]     # never read twice in a stage...
            assert set(e for e, _ in reads) <= set(e for e, _ in sw)             # ... and only for device switches
            assert int(sim.host.resident().sum()) <= cap_host
            if cap_host == E:
                assert all(v == [] for _, v in reads) and not (set(e for e, _ in reads) & seen)   # everything fits: one read each
            seen |= {e for e, _ in reads}
            n_sw += len(sw); n_rd += len(reads)
            del on_host
        assert n_rd <= n_sw
        if cap_host < E:
            assert 0 < n_rd


# ---------------------------------------------------------------------------------------------
# margin guard: admissible outcomes at near-ties
# ---------------------------------------------------------------------------------------------
def test_cache_in_use_depth_rotates_slots(oracle):
    """Root 0 (probability 1) and leaves 1..6 with probabilities 0.6 .. 0.1; four experts fit: 0, 1, 2, 3 after the
    initial fill.  One stage needs 0, 1, 4, 5, 6: plan order 0, 1 (on the device), then 4, 5, 6 (missing).
    Depth 0 (only groups that have not run are protected): 4 replaces 3 (least probable idle expert), 5 replaces 4
    (it has run and is the least probable), 6 replaces 5: one slot, every copy waits for the group before it.
    Depth 1 (the group right before a missing one is still running): 4 replaces 3; for 5 expert 4 is busy, so the
    least probable of the others goes: 2; 6 then replaces 4 (5 is busy, 4 has finished): two slots alternate."""
    E = 7
    prob = [1.0, 0.6, 0.5, 0.4, 0.3, 0.2, 0.1]
    succ_off = [0, 6] + [6] * 6
    hg = np.zeros(E, np.uint8); hg[[0, 1, 4, 5, 6]] = 1
    want = {0: [(4, [3]), (5, [4]), (6, [5])], 1: [(4, [3]), (5, [2]), (6, [4])]}
    for depth in (0, 1):
        sim = oracle.CacheSim([10] * E, prob, succ_off, list(range(1, E)), cap_experts=4, in_use=depth)
        assert sim.init_fill() == [0, 1, 2, 3]
        order, sw = sim.stage(hg)
        assert order == [0, 1, 4, 5, 6] and sw == want[depth], (depth, sw)


def test_cache_comparison_rules_textbook_reference_string(oracle):
    """The replacement rules of the paper's comparison systems (Section 5.1) on the textbook reference string
    1 2 3 4 1 2 5 1 2 3 4 5 with three frames (Belady's example: 9 faults first-in-first-out, 10 least-recently-used).
    The initial fill loads 1, 2, 3 in that order (descending probability), which is the state after the three cold
    faults; the remaining references then cost 6 and 7 switches with the victims worked out by hand:
      FIFO: 4 evicts 1, 1 evicts 2, 2 evicts 3, 5 evicts 4, (1, 2 hit), 3 evicts 1, 4 evicts 2, (5 hits)
      LRU : 4 evicts 1, 1 evicts 2, 2 evicts 3, 5 evicts 4, (1, 2 hit), 3 evicts 5, 4 evicts 1, 5 evicts 2"""
    E = 6
    prob = [0.0, 0.9, 0.8, 0.7, 0.1, 0.05]
    refs = [1, 2, 3, 4, 1, 2, 5, 1, 2, 3, 4, 5]
    want = {2: [(4, [1]), (1, [2]), (2, [3]), (5, [4]), (3, [1]), (4, [2])],
            1: [(4, [1]), (1, [2]), (2, [3]), (5, [4]), (3, [5]), (4, [1]), (5, [2])]}
    for rule in (1, 2):
        sim = oracle.CacheSim([10] * E, prob, [0] * (E + 1), [], cap_experts=3, rule=rule)
        assert sim.init_fill() == [1, 2, 3]
        log = []
        for r in refs:
            hg = np.zeros(E, np.uint8); hg[r] = 1
            order, sw = sim.stage(hg)
            assert order == [r]
            log += sw
        assert log == want[rule], (rule, log)


def test_admissible_outcomes_planted(oracle):
    from oracle import guard as G
    a = _head_only_arch(4)
    # expert 0: logits = (m0, m1, m2, 0) route over 3 classes to experts 1, 2, final
    e0 = _planted_blob(a, [[1, 0, 0], [0, 1, 0], [0, 0, 1], [0, 0, 0]], [0, 0, 0, 0])
    e1 = _planted_blob(a, [[0, 0, 0]] * 4, [1, 2, 3, 4])
    e2 = _planted_blob(a, [[0, 0, 0]] * 4, [5, 6, 7, 8])
    g = W.graph_from_lists([[1, 2, -1], [], []])
    wl = W.Workload("planted", 0, [a], [0, 0, 0], [1, .5, .5], g, 1, None, 0, 1, {}, 2)
    blobs = [e0, e1, e2]

    def img(m):
        return np.broadcast_to(np.array(m, np.float32), (2, 2, 3)).copy()

    # clear winner: class 0 by a wide gap -> one outcome, the oracle's
    out = G.admissible_outcomes(wl, blobs, img([10, 1, 2]), 0, delta=2e-2)
    assert [p.tolist() for p, _ in out] == [[0, 1]] and out[0][1].tolist() == [1, 2, 3, 4]
    # classes 0 and 1 within 1 % of the largest logit magnitude (10): both routes admissible, best first
    out = G.admissible_outcomes(wl, blobs, img([10, 9.95, 2]), 0, delta=2e-2)
    assert [p.tolist() for p, _ in out] == [[0, 1], [0, 2]] and out[1][1].tolist() == [5, 6, 7, 8]
    # a final (-1) route within the tolerance: stopping at expert 0 is admissible too
    out = G.admissible_outcomes(wl, blobs, img([10, 2, 9.9]), 0, delta=2e-2)
    assert sorted(p.tolist() for p, _ in out) == [[0, -1], [0, 1]]
    stop = [lg for p, lg in out if p.tolist() == [0, -1]][0]
    np.testing.assert_allclose(stop, [10, 2, 9.9, 0], rtol=1e-6)
    # guarded_inputs marks what it could not resolve instead of failing
    wl2 = W.config2(6, hw=32, n_experts=4, width=8, calibrated=False)
    wl2.head_bias[0] = np.zeros(16, np.float32)
    b2 = [wl2.blob(e) for e in range(4)]
    x, sub, res, redraws = G.guarded_inputs(wl2, b2, range(6), delta=10.0, max_rounds=1)    # absurd delta: nothing passes
    assert res["ambiguous"].all() and redraws == 6 and sub.tolist() == [1] * 6


# ---------------------------------------------------------------------------------------------------------------
# arranging window (paper Section 4.2 "Request arranging"): replay of which group waits and which runs
# ---------------------------------------------------------------------------------------------------------------
def _tree_cache(oracle, probs, cap):
    """root 0 -> leaves 1..n, equal sizes, capped by expert count, past its initial fill"""
    E = len(probs)
    succ_off = [0, E - 1] + [E - 1] * (E - 1)
    sim = oracle.CacheSim([100] * E, probs, succ_off, list(range(1, E)), cap_experts=cap)
    sim.init_fill()
    return sim


def test_arranging_hand_worked_schedule(oracle):
    """Root 0 and leaves 1 (probability 0.6), 2 (0.4); the cache holds two experts, so after the initial fill 0 and 1
    are on the device.  Window: a group of a missing expert waits until it has 3 requests, at most 2 steps.
    Requests r0..r5 visit [0,1] [0,2] [0,2] [0,1] [0,2] [0,2]; hand-overs: {r0,r1} {r2,r3} {r4} {r5}.
      step 0: group 0 = {r0,r1} runs.
      step 1: 0 = {r2,r3} runs; 1 = {r0} runs (on the device: no threshold); 2 = {r1}: missing, 1 < 3, age 1 < 2: waits.
      step 2: 0 = {r4} runs; 1 = {r3} runs; 2 = {r1,r2}: the oldest has waited 2 steps: runs, loaded in place of
              expert 1 (both residents have run by then; 1 has the lower usage probability).
      step 3: 0 = {r5} runs; 2 = {r4} runs (on the device now).
      step 4: 2 = {r5} runs.
    One switch.  Without the window the same arrivals alternate experts 1 and 2 in the second slot: three switches."""
    from oracle import arrange
    paths = [[0, 1], [0, 2], [0, 2], [0, 1], [0, 2], [0, 2]]
    submits = [[0, 1], [2, 3], [4], [5]]
    rec = arrange.replay(submits, paths, [0, 0, 0], {0: (0, 3, 2)}, _tree_cache(oracle, [1.0, 0.6, 0.4], 2))
    assert [r["run"] for r in rec] == [{0: [0, 1]}, {0: [2, 3], 1: [0]}, {0: [4], 1: [3], 2: [1, 2]}, {0: [5], 2: [4]}, {2: [5]}]
    assert [r["deferred"] for r in rec] == [{}, {2: [1]}, {}, {}, {}]
    assert [r["n_pending"] for r in rec] == [2, 4, 4, 2, 1]
    assert [r["switches"] for r in rec] == [[], [], [(2, [1])], [], []]
    assert [r["order"] for r in rec] == [[0], [0, 1], [0, 1, 2], [0, 2], [2]]
    plain = arrange.replay(submits, paths, [0, 0, 0], {}, _tree_cache(oracle, [1.0, 0.6, 0.4], 2))
    assert [r["deferred"] for r in plain] == [{}] * len(plain)
    assert [r["switches"] for r in plain] == [[], [(2, [1])], [(1, [2])], [(2, [1])], []]


def test_arranging_rule_cases():
    from oracle.arrange import stays_queued
    assert not stays_queued(0, 0, False, 5, 5, 5)                  # nothing queued
    assert stays_queued(2, 0, False, 0, 3, 1)                      # missing, small, young
    assert not stays_queued(3, 0, False, 0, 3, 1)                  # reached the threshold
    assert not stays_queued(2, 1, False, 0, 3, 1)                  # waited long enough
    assert not stays_queued(2, 0, True, 0, 3, 1)                   # on the device: its own threshold (none)
    assert stays_queued(2, 0, True, 4, 0, 1) and not stays_queued(2, 0, False, 4, 0, 1)
    assert not stays_queued(1, 0, False, 100, 100, 0)              # window off


@pytest.mark.parametrize("seed", range(6))
def test_arranging_invariants_random(oracle, seed):
    """Random trees, arrival sequences and windows: every request runs the stages of its path once each and in order,
    one stage per step at most; nobody waits beyond max_wait; a waiting group is small and young; with max_wait = 0
    the schedule is the plain one (every queued group runs in every step)."""
    from oracle import arrange
    rng = np.random.default_rng(100 + seed)
    n_leaves = int(rng.integers(2, 9))
    E = n_leaves + 1
    probs = [1.0] + list(np.sort(rng.random(n_leaves))[::-1] * 0.9 + 0.01)
    n = int(rng.integers(20, 120))
    paths = [[0, int(rng.integers(1, E))] if rng.random() < 0.9 else [0] for _ in range(n)]
    cuts = np.sort(rng.choice(np.arange(1, n), size=int(rng.integers(1, 8)), replace=False))
    submits = [list(range(a, b)) for a, b in zip([0] + list(cuts), list(cuts) + [n])]
    win = (int(rng.integers(0, 4)), int(rng.integers(0, 12)), int(rng.integers(0, 5)))
    cap = int(rng.integers(2, E + 1))
    rec = arrange.replay(submits, paths, [0] * E, {0: win}, _tree_cache(oracle, probs, cap))
    first_seen = {r: k for k, batch in enumerate(submits) for r in batch}
    ran = {r: [] for r in range(n)}
    for k, st in enumerate(rec):
        assert st["step"] == k and not (set(st["run"]) & set(st["deferred"]))
        for e, members in st["run"].items():
            for r in members:
                ran[r].append((k, e))
        for e, members in st["deferred"].items():
            age = k - min(first_seen[r] for r in members)
            assert age < win[2] and len(members) < max(win[0], win[1])
        assert st["n_pending"] == sum(len(m) for m in st["run"].values()) + sum(len(m) for m in st["deferred"].values())
    for r in range(n):
        assert [e for k, e in ran[r]] == paths[r]
        steps = [k for k, e in ran[r]]
        assert steps == sorted(set(steps)) and steps[0] >= first_seen[r]
        # stage i is queued from step max(first_seen, previous stage + 1) on and runs before the request's age passes max_wait
        for i, k in enumerate(steps):
            queued_from = first_seen[r] if i == 0 else steps[i - 1] + 1
            assert k <= max(queued_from, first_seen[r] + win[2])
    off = arrange.replay(submits, paths, [0] * E, {0: (win[0], win[1], 0)}, _tree_cache(oracle, probs, cap))
    assert all(not st["deferred"] for st in off)
    plain = arrange.replay(submits, paths, [0] * E, {}, _tree_cache(oracle, probs, cap))
    assert [(st["run"], st["switches"]) for st in off] == [(st["run"], st["switches"]) for st in plain]


def test_assigning_hand_worked():
    """Three executors, units of cost 5 3 3 4 2 6 1 in arrival order.  Queue times after each unit:
    5|0|0, 5|3|0, 5|3|3, 5|7|3 (the 4: queues 1 and 2 both end at 7, which is also the smallest total; the lower number
    wins), 5|7|5, 11|7|5 (the 6: queues 0 and 2 both end at 11; the lower number wins), 11|7|6."""
    from oracle.arrange import assign
    assert assign([5, 3, 3, 4, 2, 6, 1], 3) == [0, 1, 2, 1, 2, 0, 2]
    assert assign([7, 7, 7], 1) == [0, 0, 0]
    assert assign([], 4) == []
    # equal costs go round the executors in turn
    assert assign([2] * 7, 3) == [0, 1, 2, 0, 1, 2, 0]
