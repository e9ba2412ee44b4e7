"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import os
import time

import numpy as np
import pytest

import coe_workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2503_02354_amd import binding
    return binding


@pytest.fixture(scope="module")
def G():
    from oracle import guard
    return guard


from gpu_util import REL_TOL_BF16, REL_TOL_F32, assert_chain_parity, device_tensor, rel_err, run_chain_gpu  # noqa: E402


# ---------------------------------------------------------------------------------------------------------------
# regroup: bit exact
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,E,mode", [
    (0, 4, "uniform"), (1, 1, "uniform"), (63, 3, "uniform"), (255, 16, "uniform"), (256, 16, "uniform"),
    (257, 16, "holes"), (4096, 16, "uniform"), (5000, 64, "zipf"), (8192, 120, "zipf"), (16384, 64, "holes"),
    (3000, 2048, "uniform"), (4096, 32, "single"), (1000, 7, "none"),
])
def test_regroup_bit_exact(B, oracle, n, E, mode):
    rng = np.random.default_rng(n * 31 + E)
    if mode == "uniform":
        cur = rng.integers(0, E, n)
    elif mode == "holes":
        cur = rng.integers(-1, E, n); cur[rng.random(n) < 0.3] = -1
    elif mode == "zipf":
        cur = rng.choice(E, size=n, p=W.zipf_probs(E, 1.1)); cur[rng.random(n) < 0.1] = -1
    elif mode == "single":
        cur = np.full(n, E - 1)
    else:
        cur = np.full(n, -1)
    cur = cur.astype(np.int32)
    ctx = B.Context(max_requests=max(n, 1))
    got = ctx.coe_debug_regroup(cur, E)
    ctx.close()
    want = oracle.regroup(cur, E)
    assert got["n_pending"] == want["n_pending"]
    for k in ("cnt", "off", "perm"):
        assert np.array_equal(got[k], want[k]), k
    assert np.array_equal(got["inv"], want["inv"])


# ---------------------------------------------------------------------------------------------------------------
# single-expert forwards
# ---------------------------------------------------------------------------------------------------------------
def _forward_case(B, oracle, arch, n, seed, tol, max_batch=0):
    blob = W.make_expert_blob(arch, seed, 0)
    x = W.make_inputs(arch, seed, range(n))
    ctx = B.Context(max_requests=max(n, 1), max_batch=max_batch)
    aid = ctx.coe_register_arch(arch)
    assert ctx.coe_arch_blob_bytes(aid) == blob.nbytes == W.blob_layout(arch)[1]
    ctx.coe_register_expert(0, aid, blob, 1.0)
    dev = device_tensor(x)
    got = ctx.coe_debug_forward(0, n, dev.data_ptr())
    ctx.close()
    want = np.stack([oracle.forward(arch, blob, x[i]) for i in range(n)])
    err = rel_err(got, want)
    assert err.max() <= tol, err.max()


def test_forward_tiny_cnn_fp32(B, oracle):
    _forward_case(B, oracle, W.tiny_cnn(4, 64), 9, 11, REL_TOL_F32, max_batch=4)


def test_forward_resnet18_bf16(B, oracle):
    _forward_case(B, oracle, W.resnet18(16, 64, W.DT_BF16, 32), 7, 12, REL_TOL_BF16, max_batch=3)


def test_forward_resnet18_fp32(B, oracle):
    _forward_case(B, oracle, W.resnet18(10, 48, W.DT_F32, 16), 5, 13, REL_TOL_F32)


def test_forward_resnet50_bf16(B, oracle):
    _forward_case(B, oracle, W.resnet50(12, 64, W.DT_BF16, 32), 5, 14, REL_TOL_BF16)


def test_forward_resnet18_bf16_full_width_ragged(B, oracle):
    # real channel counts (64..512), odd spatial size so tiles end ragged (input 72 -> 36 -> 18, 9, 5, 3)
    _forward_case(B, oracle, W.resnet18(16, 72, W.DT_BF16, 64), 3, 15, REL_TOL_BF16)


def _conv_pair_arch(H, Wd, C, K, R, stride, pad, ncls=8):
    """conv(RxR, stride) + ReLU, then conv3x3 with the first output as residual + ReLU, then the head: a permuted or
    misplaced output tile of the first conv changes the second conv's result."""
    p = W._Prog(H, Wd, C)
    p.conv(0, 1, K, R, stride, pad, W.ACT_RELU)
    p.conv(1, 2, K, 3, 1, 1, W.ACT_RELU, res=1, gain=0.5)
    p.head(2, ncls)
    return W.Arch("conv_pair", W.DT_BF16, H, Wd, C, ncls, np.array(p.layers, dtype=np.int32), p.gains)


@pytest.mark.parametrize("H,Wd,C,K,R,stride,pad,n", [
    (14, 14, 64, 128, 3, 1, 1, 5),      # 128-wide filter tile, rows end ragged (980 rows)
    (9, 11, 32, 64, 3, 1, 1, 3),        # 64-wide filter tile, one partial row tile
    (10, 10, 96, 32, 3, 2, 1, 4),       # 32-wide filter tile, stride 2, C = 3 reduction blocks
    (16, 12, 64, 256, 1, 1, 0, 6),      # 1x1
    (15, 15, 128, 128, 1, 2, 0, 3),     # 1x1 stride 2 (shortcut conv)
    (7, 7, 512, 512, 3, 1, 1, 11),      # late-stage shape: 539 rows, 4 filter tiles, long reduction
    (56, 56, 64, 64, 3, 1, 1, 2),       # first-stage shape: many row tiles across the XCD remap
    (5, 5, 32, 96, 5, 1, 2, 2),         # 5x5 window, K = 96 -> 32-wide tiles
])
def test_conv_mfma_shapes(B, oracle, H, Wd, C, K, R, stride, pad, n):
    _forward_case(B, oracle, _conv_pair_arch(H, Wd, C, K, R, stride, pad), n, 100 + H + K, REL_TOL_BF16)


@pytest.mark.parametrize("H,Wd,C,K,R,stride,pad,n", [
    (37, 46, 3, 64, 7, 2, 3, 3),        # stem shape at an odd size: ragged 16x16 tiles on both axes
    (37, 45, 3, 64, 7, 2, 3, 3),        # odd row length in elements: the stem kernel declines, the plain kernel runs
    (224, 224, 3, 64, 7, 2, 3, 2),      # the real stem: 7x7 tiles per image, several tiles per workgroup
    (30, 30, 4, 32, 3, 1, 1, 2),        # C=4, stride 1, 32 filters
    (20, 33, 6, 64, 5, 1, 2, 2),        # C=6: 30-element window rows -> 4 chunks per row
    (64, 64, 3, 32, 7, 2, 3, 40),       # many images: the tile loop wraps around the grid
])
def test_conv_small_channel_shapes(B, oracle, H, Wd, C, K, R, stride, pad, n):
    _forward_case(B, oracle, _conv_pair_arch(H, Wd, C, K, R, stride, pad), n, 200 + H + K, REL_TOL_BF16)


# ---------------------------------------------------------------------------------------------------------------
# whole chains
# ---------------------------------------------------------------------------------------------------------------
def test_config1_full_size(B, oracle, G):
    """Config 1 as specified: 4 fp32 tiny-CNN experts, 256 requests of 3x64x64, expert 0 routes over classes 0-2."""
    wl = W.config1(calibrated=False)
    G.calibrate_workload(wl, n_cal=64)
    blobs = [wl.blob(e) for e in range(4)]
    x, sub, want, redraws = G.guarded_inputs(wl, blobs, range(wl.n_requests))
    assert redraws < 26
    got = run_chain_gpu(B, wl, blobs, x, max_batch=100)
    assert_chain_parity(got, want, REL_TOL_F32)
    leaves = np.bincount(want["path"][:, 1], minlength=4)[1:]
    assert leaves.min() > 20, leaves                                 # calibration spreads the routes
    # regroup of the second stage equals the oracle's stable regroup of the routed ids
    assert [s[1].n_groups for s in got["stats"][:2]] == [1, 3]


def _config2_small(n=96, hw=64, E=6, width=32):
    return W.config2(n, hw=hw, n_experts=E, width=width, calibrated=False)


def test_config2_small_chain(B, oracle, G):
    wl = _config2_small()
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(wl.graph.n_experts)]
    x, sub, want, redraws = G.guarded_inputs(wl, blobs, range(wl.n_requests))
    got = run_chain_gpu(B, wl, blobs, x, max_batch=20)
    assert_chain_parity(got, want, REL_TOL_BF16)
    assert len(set(want["path"][:, 1].tolist())) >= 3
    # schedule independence on the GPU: other batch size, arrival in pieces, host inputs: identical routes and logits
    got2 = run_chain_gpu(B, wl, blobs, x, max_batch=7, arrival=25, on_device=False)
    assert np.array_equal(got2["path"], got["path"])
    assert rel_err(got2["logits"], got["logits"]).max() <= 1e-6


def test_regroup_inside_step_matches_oracle(B, oracle, G):
    wl = _config2_small(n=80)
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(wl.graph.n_experts)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(80))
    ctx = B.Context(max_requests=80, max_stages=2, max_batch=16)
    B.setup_workload(ctx, wl, blobs)
    dev = device_tensor(x)
    ctx.coe_submit(80, dev.data_ptr(), True)
    ctx.coe_step()
    r1 = ctx.coe_debug_last_regroup(80)
    assert r1["perm"].tolist() == list(range(80)) and r1["cnt"][0] == 80           # single root: identity
    ctx.coe_step()
    r2 = ctx.coe_debug_last_regroup(80)
    ref = oracle.regroup(want["path"][:, 1], wl.graph.n_experts)
    for k in ("cnt", "off", "perm", "inv"):
        assert np.array_equal(r2[k], ref[k]), k
    rc, _ = ctx.coe_step()
    assert rc == B.COE_DONE
    ctx.close()


def test_request_splitting_matches_the_oracle_chunk_table(B, oracle, G):
    """Request splitting (Section 4.2): the batches the library launched in a step, {expert, first row, count} each, against
    the oracle's split of the same regrouped stage, batch by batch, for several maximum batch sizes."""
    wl = _config2_small(n=80)
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(wl.graph.n_experts)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(80))
    dev = device_tensor(x)
    for max_batch in (1, 3, 7, 16, 33, 80):
        ctx = B.Context(max_requests=80, max_stages=2, max_batch=max_batch, group_small=-1)
        B.setup_workload(ctx, wl, blobs)
        ctx.coe_submit(80, dev.data_ptr(), True)
        for stage in range(2):
            rc, st = ctx.coe_step()
            got = ctx.coe_debug_last_chunks()
            keys = want["path"][:, stage] if stage else np.zeros(80, np.int32)
            rg = oracle.regroup(keys, wl.graph.n_experts)
            order = [e for e in range(wl.graph.n_experts) if rg["cnt"][e] > 0]      # everything resident: ascending id
            ref = oracle.split(rg["off"], order, max_batch)
            assert got.tolist() == ref.tolist(), (max_batch, stage)
            assert st.n_chunks == len(ref)
        ctx.close()


def test_capped_cache_switches_match_policy_and_results_do_not_change(B, oracle, G):
    """Config-3 structure at small scale: Zipf leaves, capped cache, requests arriving in batches."""
    wl = W.config3(120, hw=64, n_experts=10, width=16, cap=4, arrival_batch=30, calibrated=False)
    G.calibrate_workload(wl, n_cal=64, targets={0: W.zipf_probs(9, 1.1)})
    blobs = [wl.blob(e) for e in range(10)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(120))
    got = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=30)
    assert_chain_parity(got, want, REL_TOL_BF16)
    # replay the oracle's cache simulator over the same per-step group sets
    nbytes = [blobs[e].nbytes for e in range(10)]
    sim = oracle.CacheSim(nbytes, wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_experts=4)
    log = [(e, []) for e in sim.init_fill()]
    pend = {}                                                       # request -> expert it waits for
    nxt = 0
    for rc, st in got["stats"]:
        if nxt < 120:
            for r in range(nxt, nxt + 30):
                pend[r] = 0
            nxt += 30
        if not pend:
            break
        hg = np.zeros(10, np.uint8); hg[list(set(pend.values()))] = 1
        order, sw = sim.stage(hg)
        log += sw
        assert st.n_groups == len(order) and st.n_misses == len(sw)
        new = {}
        for r, e in pend.items():
            stage = want["path"][r].tolist().index(e)
            if stage + 1 < want["path"].shape[1] and want["path"][r, stage + 1] >= 0:
                new[r] = int(want["path"][r, stage + 1])
        pend = new
    assert got["switch_log"] == log
    assert len(log) > 6                                             # the cap really forces switches
    # uncapped and cap=2 (every group a switch) give the same routes and logits
    for cap in (0, 2):
        g2 = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=30, cap_experts=cap)
        assert np.array_equal(g2["path"], got["path"])
        assert rel_err(g2["logits"], got["logits"]).max() <= 1e-6


@pytest.mark.parametrize("rule,depth,host_cap", [(0, 0, 6), (0, 2, 5), (1, 1, 4)])
def test_host_tier_serves_switches_from_a_file(B, oracle, G, tmp_path, rule, depth, host_cap):
    """Third storage level (Section 5.1: CPU memory as a cache in front of the SSD): every expert lives in a backing file, at
    most host_cap of them in pinned host memory, four on the device.  Results and the device's switch log equal those of the
    run that keeps every expert in host memory, the reads from the file equal the oracle's two-level replay, and the file is
    gone after the context."""
    wl = W.config3(120, hw=64, n_experts=10, width=16, cap=4, arrival_batch=30, calibrated=False)
    G.calibrate_workload(wl, n_cal=64, targets={0: W.zipf_probs(9, 1.1)})
    blobs = [wl.blob(e) for e in range(10)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(120))
    plain = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=30, eviction=rule, prefetch_depth=depth)
    assert_chain_parity(plain, want, REL_TOL_BF16)
    assert plain["host_log"] == []
    path = str(tmp_path / "experts.bin")
    got = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=30, eviction=rule, prefetch_depth=depth, host_tier=(host_cap, path),
                        keep=True)
    ctx = got.pop("ctx")
    assert os.path.getsize(path) >= sum(b.nbytes for b in blobs)
    assert np.array_equal(got["path"], plain["path"]) and np.array_equal(got["logits"], plain["logits"])
    assert got["switch_log"] == plain["switch_log"]
    # the oracle's replay of both levels over the same per-step group sets
    sim = oracle.TieredCacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_device=4,
                                cap_host=host_cap, rule=rule, in_use=depth)
    loaded, reads = sim.init_fill()
    log = [(e, []) for e in loaded]
    n_init = len(reads)
    pend, nxt, per_step = {}, 0, []
    for rc, st in got["stats"]:
        if nxt < 120:
            for r in range(nxt, nxt + 30):
                pend[r] = 0
            nxt += 30
        if not pend:
            break
        hg = np.zeros(10, np.uint8); hg[list(set(pend.values()))] = 1
        order, sw, rd = sim.stage(hg)
        log += sw
        reads += rd
        per_step.append(len(rd))
        assert st.n_misses == len(sw) and st.n_host_misses == len(rd) + (n_init if len(per_step) == 1 else 0)
        assert st.bytes_read == st.n_host_misses * blobs[0].nbytes
        new = {}
        for r, e in pend.items():
            stage = want["path"][r].tolist().index(e)
            if stage + 1 < want["path"].shape[1] and want["path"][r, stage + 1] >= 0:
                new[r] = int(want["path"][r, stage + 1])
        pend = new
    assert got["switch_log"] == log and got["host_log"] == reads
    assert sum(per_step) > 0 and len(reads) < n_init + len(log)        # the host level both misses and hits
    with pytest.raises(B.CoEError):                                   # direct forwards are served from the device only
        missing = int(np.nonzero(~ctx.coe_debug_resident())[0][0])
        ctx.coe_debug_forward(missing, 1, device_tensor(x[:1]).data_ptr())
    ctx.close()
    assert not os.path.exists(path)


def test_host_tier_with_two_architectures(B, oracle, G, tmp_path):
    """Two blob sizes, so two slot classes on both levels: 18 experts in the file, 8 in host memory, 5 on the device, requests
    arriving in five batches.  Same bits and the same device switches as without the file; the reads are what the lower level's
    policy does when it is asked for every device switch in turn."""
    n, arrival = 120, 24
    wl = W.config4(n, hw=64, tiers=(3, 6, 9), width=16, fan=(3, 2), calibrated=False)
    G.calibrate_workload(wl, n_cal=32)
    E = wl.graph.n_experts
    blobs = [wl.blob(e) for e in range(E)]
    assert len(set(b.nbytes for b in blobs)) == 2
    x = wl.inputs(range(n))
    kw = dict(max_batch=32, arrival=arrival, cap_experts=5, prefetch_depth=1)
    plain = run_chain_gpu(B, wl, blobs, x, wl.first_expert, **kw)
    path = str(tmp_path / "experts.bin")
    got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, host_tier=(8, path), **kw)
    assert np.array_equal(got["path"], plain["path"]) and np.array_equal(got["logits"], plain["logits"])
    assert got["switch_log"] == plain["switch_log"] and len(got["switch_log"]) > 15
    host = oracle.CacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_experts=8)
    reads = [(e, []) for e in host.init_fill()]
    for e, _ in got["switch_log"]:
        need = np.zeros(E, np.uint8); need[e] = 1
        reads += host.stage(need)[1]
    assert got["host_log"] == reads and len(reads) > 8 + 5
    stats = [st for rc, st in got["stats"] if rc == B.COE_OK]
    assert sum(st.n_host_misses for st in stats) == len(reads)
    assert sum(st.bytes_read for st in stats) == sum(blobs[e].nbytes for e, _ in reads)
    assert all(st.n_device_allocs == 0 for st in stats)
    assert not os.path.exists(path)


def test_host_tier_read_failure_is_an_error_not_a_hang(B, tmp_path):
    """A backing file that has lost its contents: the step that needs a read from it fails with COE_EIO, the loader thread's
    queue drains, and the context can still be destroyed."""
    wl = W.config3(40, hw=64, n_experts=8, width=16, cap=3, arrival_batch=40, calibrated=False)
    blobs = [wl.blob(e) for e in range(8)]
    x = wl.inputs(range(40))
    path = str(tmp_path / "experts.bin")
    ctx = B.Context(max_requests=40, max_stages=wl.max_stages, max_batch=16, cache_cap_experts=3)
    ctx.coe_set_host_tier(4, path)
    B.setup_workload(ctx, wl, blobs)
    os.truncate(path, 0)
    ctx.coe_submit(40, x, False, None)
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_step()
    assert ei.value.code == B.COE_EIO
    ctx.close()
    assert not os.path.exists(path)


def test_host_tier_argument_checks(B, tmp_path):
    ctx = B.Context(max_requests=4)
    for cap, path in ((0, str(tmp_path / "a")), (2, ""), (2, str(tmp_path / "no_such_dir" / "a"))):
        with pytest.raises(B.CoEError):
            ctx.coe_set_host_tier(cap, path)
    ctx.coe_set_host_tier(2, str(tmp_path / "b"))
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_set_host_tier(2, str(tmp_path / "c"))
    assert ei.value.code == B.COE_ESTATE
    ctx.close()
    assert not os.path.exists(tmp_path / "b")


def test_config4_small_dag(B, oracle, G):
    """Three-stage DAG, two architectures, shared downstream experts, skewed first experts."""
    wl = W.config4(150, hw=64, tiers=(3, 6, 9), width=16, fan=(3, 2), calibrated=False)
    G.calibrate_workload(wl, n_cal=32)
    E = wl.graph.n_experts
    blobs = [wl.blob(e) for e in range(E)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(150))
    got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, max_batch=32)
    assert_chain_parity(got, want, REL_TOL_BF16)
    assert np.all(got["path"][:, 2] >= 0)


# ---------------------------------------------------------------------------------------------------------------
# error paths and degenerate inputs (forced from the host; no kernel misbehaves)
# ---------------------------------------------------------------------------------------------------------------
def test_error_codes_and_empty_inputs(B):
    wl = W.config1(8, hw=16, calibrated=False)
    blobs = [wl.blob(e) for e in range(4)]
    ctx = B.Context(max_requests=8, max_stages=2)
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_submit(1, np.zeros((1, 16, 16, 3), np.float32), False)
    assert ei.value.code == B.COE_ESTATE                             # graph not set
    aid = ctx.coe_register_arch(wl.archs[0])
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_register_expert(0, aid, blobs[0][:-256], 1.0)
    assert ei.value.code == B.COE_EINVAL                             # wrong blob size
    for e in range(4):
        ctx.coe_register_expert(e, aid, blobs[e], 0.5)
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_register_expert(1, aid, blobs[1], 0.5)
    assert ei.value.code == B.COE_EINVAL                             # twice
    bad = W.graph_from_lists([[1, 2, 3, 1, 2], [], [], []])          # 5 routes > 4 classes
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_set_dependency_graph(bad.succ_off, bad.succ)
    assert ei.value.code == B.COE_EGRAPH
    deep = W.graph_from_lists([[1], [2], [3], []])                   # depth 4 > max_stages 2
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_set_dependency_graph(deep.succ_off, deep.succ)
    assert ei.value.code == B.COE_ERANGE
    ctx.coe_set_dependency_graph(wl.graph.succ_off, wl.graph.succ)
    rc, _ = ctx.coe_step()
    assert rc == B.COE_DONE                                          # nothing submitted
    assert ctx.coe_submit(0, None, False) == 0                       # empty submit is fine
    ids, logits, path = ctx.coe_collect(8)
    assert len(ids) == 0
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_submit(9, np.zeros((9, 16, 16, 3), np.float32), False)
    assert ei.value.code == B.COE_ERANGE                             # store full
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_submit(1, np.zeros((1, 16, 16, 3), np.float32), False, np.array([7], np.int32))
    assert ei.value.code == B.COE_EINVAL                             # unknown first expert
    # the context is still usable
    x = wl.inputs(range(3))
    assert ctx.coe_submit(3, x, False) == 0
    while ctx.coe_step()[0] != B.COE_DONE:
        pass
    ids, logits, path = ctx.coe_collect(8)
    assert ids.tolist() == [0, 1, 2] and np.all(path[:, 0] == 0)
    # ids keep counting after the store drained
    assert ctx.coe_submit(2, x[:2], False) == 3
    ctx.close()
    # an expert larger than the cache cap cannot run
    ctx = B.Context(max_requests=8, max_stages=2, cache_cap_bytes=1000)
    B.setup_workload(ctx, wl, blobs)
    ctx.coe_submit(2, x[:2], False)
    with pytest.raises(B.CoEError) as ei:
        ctx.coe_step()
    assert ei.value.code == B.COE_ENOMEM
    ctx.close()


# ---------------------------------------------------------------------------------------------------------------
# convolution kernels element by element (appended: the full output tensor, not only pooled logits)
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,H,Wd,C,K,R,stride,pad,use_res,act", [
    (3, 14, 14, 64, 128, 3, 1, 1, True, 1),       # MFMA, 128-wide tiles, residual
    (2, 20, 17, 64, 64, 3, 1, 1, False, 1),       # MFMA, 64-wide tiles, ragged rows
    (5, 9, 9, 32, 96, 3, 2, 1, True, 0),          # MFMA, 32-channel steps, stride 2, no activation
    (40, 8, 8, 128, 256, 1, 1, 0, False, 2),      # MFMA 1x1 with GELU, 2560 rows
    (2, 33, 30, 3, 64, 7, 2, 3, False, 1),        # stem kernel
    (2, 12, 12, 16, 24, 3, 1, 1, True, 1),        # plain kernel (bf16)
    (21, 57, 57, 64, 256, 1, 1, 0, True, 1),      # large 1x1: 68229 rows (ragged), two filter tiles per row tile, residual
    (11, 57, 57, 32, 512, 1, 1, 0, False, 2),     # one 32-channel step, four filter tiles per row tile, GELU
    (6, 57, 57, 64, 256, 3, 2, 1, False, 1),      # 3x3 stride 2 at an odd size
    (3, 28, 28, 64, 64, 3, 1, 1, True, 3),        # SiLU: slab kernel with residual (detector-shaped experts)
    (4, 14, 14, 256, 128, 1, 1, 0, False, 3),     # SiLU: 1x1
    (3, 20, 20, 32, 32, 3, 1, 1, True, 3),        # SiLU: 32 filters (register-staged kernel)
    (2, 40, 40, 3, 32, 6, 2, 2, False, 3),        # SiLU: 6x6 stride-2 stem, 32 filters
    (5, 14, 14, 128, 96, 1, 1, 0, False, 0),      # detection output: 96 = 3 anchors x 32
])
def test_conv_elementwise_bf16(B, oracle, n, H, Wd, C, K, R, stride, pad, use_res, act):
    rng = np.random.default_rng(n * 1000 + H * 10 + K)
    q = lambda a: W.f32_to_bf16_bits(a.astype(np.float32))
    xb = q(rng.standard_normal((n, H, Wd, C))).reshape(n, H, Wd, C)
    wb = q(rng.standard_normal((K, R, R, C)) * np.sqrt(2.0 / (R * R * C))).reshape(K, R, R, C)
    bias = (0.1 * rng.standard_normal(K)).astype(np.float32)
    P = (H + 2 * pad - R) // stride + 1; Q = (Wd + 2 * pad - R) // stride + 1
    rb = q(rng.standard_normal((n, P, Q, K))).reshape(n, P, Q, K) if use_res else None
    ctx = B.Context(max_requests=1)
    got, cls = ctx.coe_debug_conv(1, xb, wb, bias, rb, stride, pad, act)
    ctx.close()
    xf, wf = W.bf16_bits_to_f32(xb).reshape(xb.shape), W.bf16_bits_to_f32(wb).reshape(wb.shape)
    rf = None if rb is None else W.bf16_bits_to_f32(rb).reshape(rb.shape)
    want = np.stack([oracle.conv2d(xf[i], wf, bias, None if rf is None else rf[i], stride, pad, act, 1) for i in range(n)])
    g = W.bf16_bits_to_f32(got).reshape(got.shape)
    # both sides round the same fp32-epilogue value to bf16; fp32 vs fp64 accumulation may flip a rounding now and then
    # (one bf16 ulp), and where the terms cancel to almost nothing the fp32 accumulation error itself (terms are O(1),
    # up to ~1e3 of them: ~1e-5 absolute) is all that is left
    ulp = np.maximum(np.abs(want) * 2.0 ** -7, 1e-5)
    worst = np.unravel_index(np.argmax(np.abs(g - want) / ulp), g.shape)
    assert np.all(np.abs(g - want) <= ulp), (worst, float(g[worst]), float(want[worst]), int(np.sum(np.abs(g - want) > ulp)))
    assert np.mean(g == want) > 0.995


# ---------------------------------------------------------------------------------------------------------------
# transformer-shaped experts: each token op element by element, then whole forwards
# ---------------------------------------------------------------------------------------------------------------
def _token_op_arch(T, C, words, out_c, ncls=4):
    """One token op on the raw input [T][1][C], then a pooled head so the program is complete."""
    p = W._Prog(T, 1, C)
    p.raw([words[0], 0, 1, -1] + list(words[1:]))
    p.shape[1] = (T if words[0] != W.OP_TOKENS else T + 1, 1, out_c)
    p.head(1, ncls)
    return W.Arch("token_op", W.DT_BF16, T, 1, C, ncls, np.array(p.layers, dtype=np.int32), p.gains)


def _layer0(B, arch, blob, x, shape):
    n = x.shape[0]
    ctx = B.Context(max_requests=n, max_batch=n)
    aid = ctx.coe_register_arch(arch)
    ctx.coe_register_expert(0, aid, blob, 1.0)
    dev = device_tensor(x)
    got = ctx.coe_debug_layer_output(0, n, dev.data_ptr(), 0, (n,) + shape, np.uint16)
    ctx.close()
    return W.bf16_bits_to_f32(got).reshape(got.shape)


def _assert_bf16_close(g, want, floor):
    """Both sides round an fp32 (GPU) / fp64 (oracle) value to bf16: equal except for rounding flips of one ulp."""
    ulp = np.maximum(np.abs(want) * 2.0 ** -7, floor)
    bad = np.abs(g - want) > ulp
    worst = np.unravel_index(np.argmax(np.abs(g - want) / ulp), g.shape)
    assert not bad.any(), (worst, float(g[worst]), float(want[worst]), int(bad.sum()))


@pytest.mark.parametrize("T,D,heads,n", [(197, 128, 2, 3), (32, 64, 1, 2), (50, 192, 3, 2), (224, 64, 1, 1), (1, 64, 1, 2)])
def test_attention_elementwise(B, oracle, T, D, heads, n):
    arch = _token_op_arch(T, 3 * D, [W.OP_ATTENTION, D, 0, 0, 0, 0, 0, heads, 0], D)
    blob = W.make_expert_blob(arch, 31, 0)
    x = W.make_inputs(arch, 31, range(n)).reshape(n, T, 3 * D)
    g = _layer0(B, arch, blob, x, (T, 1, D)).reshape(n, T, D)
    xf = W.bf16_bits_to_f32(x).reshape(n, T, 3 * D)
    want = np.stack([oracle.attention(xf[i], heads, 1) for i in range(n)])
    # weights are bf16(e) on both sides; expf vs exp may flip a weight's rounding: 2^-9 relative on one term
    _assert_bf16_close(g, want, 2e-3)
    assert np.mean(g == want) > 0.98


@pytest.mark.parametrize("T,D,n", [(197, 768, 2), (5, 66, 3), (64, 2048, 1)])
def test_layernorm_elementwise(B, oracle, T, D, n):
    arch = _token_op_arch(T, D, [W.OP_LAYERNORM, D, 0, 0, 0, 0, 0, 0, 0], D)
    blob = W.make_expert_blob(arch, 32, 0)
    x = W.make_inputs(arch, 32, range(n)).reshape(n, T, D)
    g = _layer0(B, arch, blob, x, (T, 1, D)).reshape(n, T, D)
    xf = W.bf16_bits_to_f32(x).reshape(n, T, D)
    gamma, beta = W.blob_tensor(arch, blob, 0, "gamma"), W.blob_tensor(arch, blob, 0, "beta")
    want = np.stack([oracle.layernorm(xf[i], gamma, beta, 1) for i in range(n)])
    _assert_bf16_close(g, want, 1e-5)
    assert np.mean(g == want) > 0.995


def test_tokens_elementwise(B, oracle):
    T0, D, n = 49, 72, 3
    arch = _token_op_arch(T0, D, [W.OP_TOKENS, D, 0, 0, 0, 0, 0, 0, 0], D)
    blob = W.make_expert_blob(arch, 33, 0)
    x = W.make_inputs(arch, 33, range(n)).reshape(n, T0, D)
    g = _layer0(B, arch, blob, x, (T0 + 1, 1, D)).reshape(n, T0 + 1, D)
    xf = W.bf16_bits_to_f32(x).reshape(n, T0, D)
    cls, pos = W.blob_tensor(arch, blob, 0, "cls"), W.blob_tensor(arch, blob, 0, "pos")
    want = np.stack([oracle.tokens(xf[i], cls, pos, 1) for i in range(n)])
    assert np.array_equal(g, want)          # one exact fp32 add, one rounding: no room for a difference


def test_patch_embedding_elementwise(B, oracle):
    # 16x16 patches of a 3-channel image as one GEMM over gathered rows (red = 768), ragged last tile (3*4*4 = 48 rows)
    hw, patch, K, n = 64, 16, 96, 3
    p = W._Prog(hw, hw, 3)
    p.conv(0, 1, K, patch, patch, 0, W.ACT_NONE)
    p.head(1, 4)
    arch = W.Arch("patch", W.DT_BF16, hw, hw, 3, 4, np.array(p.layers, dtype=np.int32), p.gains)
    blob = W.make_expert_blob(arch, 34, 0)
    x = W.make_inputs(arch, 34, range(n)).reshape(n, hw, hw, 3)
    g = _layer0(B, arch, blob, x, (hw // patch, hw // patch, K))
    xf = W.bf16_bits_to_f32(x).reshape(n, hw, hw, 3)
    w, b = W.blob_tensor(arch, blob, 0, "w"), W.blob_tensor(arch, blob, 0, "b")
    want = np.stack([oracle.conv2d(xf[i], w, b, None, patch, 0, 0, 1) for i in range(n)])
    _assert_bf16_close(g, want, 1e-5)
    assert np.mean(g == want) > 0.995


def test_forward_vit_small_bf16(B, oracle):
    # 4 blocks, 2 heads of 64, 17 tokens: every op of the transformer program once through the library's dispatch
    _forward_case(B, oracle, W.vit(6, 32, 8, 128, 4, 2, 256, W.DT_BF16), 5, 35, REL_TOL_BF16, max_batch=3)


def test_forward_vit_base_shape_bf16(B, oracle):
    # ViT-B/16 geometry (197 tokens: ragged 32-key blocks; 12 heads; red 768) with 2 blocks to keep the oracle quick
    _forward_case(B, oracle, W.vit(8, 224, 16, 768, 2, 12, 3072, W.DT_BF16), 3, 36, REL_TOL_BF16)


# ---------------------------------------------------------------------------------------------------------------
# detector-shaped experts: concatenation, upsampling, the detection read-out, whole forwards, a classifier -> detector chain
# ---------------------------------------------------------------------------------------------------------------
def test_concat_and_upsample_elementwise(B, oracle):
    n, H, Wd, C = 3, 5, 7, 16
    for op in ("concat", "upsample"):
        p = W._Prog(H, Wd, C)
        if op == "concat":
            p.concat(0, 0, 1)
            shape = (H, Wd, 2 * C)
        else:
            p.upsample(0, 1)
            shape = (2 * H, 2 * Wd, C)
        p.head(1, 4)
        arch = W.Arch(op, W.DT_BF16, H, Wd, C, 4, np.array(p.layers, dtype=np.int32), p.gains)
        blob = W.make_expert_blob(arch, 41, 0)
        x = W.make_inputs(arch, 41, range(n)).reshape(n, H, Wd, C)
        g = _layer0(B, arch, blob, x, shape)
        xf = W.bf16_bits_to_f32(x).reshape(n, H, Wd, C)
        want = np.stack([oracle.concat(xf[i], xf[i]) if op == "concat" else oracle.upsample2(xf[i]) for i in range(n)])
        assert np.array_equal(g, want), op              # pure data movement: bit for bit


def test_detection_readout_elementwise(B, oracle):
    # detection maps are the raw input here: 6x5 positions, 2 anchors, 11 classes -> 32 channels; a second, coarser map through
    # an identity-free path is covered by the whole-forward tests below
    n, H, Wd, anchors, ncls = 4, 6, 5, 2, 11
    C = anchors * (5 + ncls)
    p = W._Prog(H, Wd, C)
    p.det_head(0, -1, ncls, anchors)
    arch = W.Arch("readout", W.DT_BF16, H, Wd, C, ncls, np.array(p.layers, dtype=np.int32), p.gains)
    blob = W.make_expert_blob(arch, 42, 0)
    x = W.make_inputs(arch, 42, range(n)).reshape(n, H, Wd, C)
    ctx = B.Context(max_requests=n, max_batch=n)
    aid = ctx.coe_register_arch(arch)
    ctx.coe_register_expert(0, aid, blob, 1.0)
    got = ctx.coe_debug_forward(0, n, device_tensor(x).data_ptr())
    ctx.close()
    xf = W.bf16_bits_to_f32(x).reshape(n, H, Wd, C)
    want = np.stack([oracle.det_head([xf[i]], anchors, ncls) for i in range(n)])
    np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-7)     # fp32 sigmoids against fp64 ones


def test_forward_detector_small_bf16(B, oracle):
    _forward_case(B, oracle, W.detector(27, 64, 16, 3, W.DT_BF16), 6, 43, REL_TOL_BF16, max_batch=4)


def test_forward_detector_full_shape_bf16(B, oracle):
    # the detector at the size the classifier -> detector workload uses: 224x224 input, width 64, detection maps 28x28 and 14x14
    _forward_case(B, oracle, W.detector(27, 224, 64, 3, W.DT_BF16), 3, 44, REL_TOL_BF16)


def test_classifier_to_detector_chain(B, oracle, G):
    """The paper's own workload shape (Section 5.1) at small scale: ResNet-18-shaped classifiers route to detector-shaped
    experts that several classifiers share; a request's result is its detector's read-out.  Routes bit-exact, logits within
    tolerance, also with a capped cache (two slot classes in the expert arena) and with arrivals in pieces."""
    n = 96
    wl = W.config6(n, hw=64, n_classifiers=3, n_detectors=5, fan=4, width=16, det_width=16, calibrated=False)
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(wl.graph.n_experts)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    assert not want["ambiguous"].any()
    got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, max_batch=32)
    assert_chain_parity(got, want, REL_TOL_BF16)
    assert len(set(want["path"][:, 1].tolist())) >= 3 and np.all(want["path"][:, 1] >= 3)      # every request ends in a detector
    capped = run_chain_gpu(B, wl, blobs, x, wl.first_expert, max_batch=20, cap_experts=3, arrival=24, prefetch_depth=1)
    assert np.array_equal(capped["path"], got["path"]) and np.array_equal(capped["logits"], got["logits"])
    assert sum(st.n_misses for rc, st in capped["stats"] if rc == B.COE_OK) > 0


def test_forward_is_deterministic_and_batch_independent(B):
    """Full-width ResNet-18 at 224x224, 512 requests (thousands of tiles per conv launch, every kernel at its bench
    shape): repeated runs give the same bits, and a request's logits do not depend on how many requests run with it.
    Guards the LDS hand-over between pipeline stages of the conv kernels (a stale or early-overwritten operand stage
    shows up as a handful of wrong tiles per run)."""
    import torch
    arch = W.resnet18(16, 224, W.DT_BF16, 64)
    blob = W.make_expert_blob(arch, 77, 0)
    n = 512
    x = W.make_inputs(arch, 77, range(n))
    ctx = B.Context(max_requests=n, max_batch=n)
    aid = ctx.coe_register_arch(arch)
    ctx.coe_register_expert(0, aid, blob, 1.0)
    dev = device_tensor(x)
    runs = [ctx.coe_debug_forward(0, n, dev.data_ptr()) for _ in range(4)]
    small = ctx.coe_debug_forward(0, 48, dev.data_ptr())
    ctx.close()
    assert np.isfinite(runs[0]).all()
    for r in runs[1:]:
        assert np.array_equal(r, runs[0])
    assert np.array_equal(small, runs[0][:48])


# ---------------------------------------------------------------------------------------------------------------
# small groups sharing launches: same bits as one launch sequence per group, with and without a capped cache
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cap", [0, 5])
def test_grouped_launches_give_the_same_bits(B, oracle, G, cap):
    """Full-width ResNet-18-shaped experts (every conv has a multiple of 64 filters, so the architecture is
    groupable), 1 root -> 15 leaves, 160 requests: the leaf groups hold ~10 requests each and share launches.
    Grouping must not change a bit, must respect the cache policy's switch log, and must still match the oracle."""
    wl = W.config2(160, hw=64, n_experts=16, width=64, calibrated=False)
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(16)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(160))
    one = run_chain_gpu(B, wl, blobs, x, max_batch=128, cap_experts=cap, group_small=-1)
    grp = run_chain_gpu(B, wl, blobs, x, max_batch=128, cap_experts=cap)
    assert sum(st.n_grouped for rc, st in one["stats"]) == 0
    stats = [st for rc, st in grp["stats"] if rc == B.COE_OK]
    assert stats[1].n_grouped >= 8 and 1 <= stats[1].n_group_sets < stats[1].n_grouped     # several groups per launch set
    assert np.array_equal(one["path"], grp["path"])
    assert np.array_equal(one["logits"], grp["logits"])
    assert one["switch_log"] == grp["switch_log"]
    assert [st.n_chunks for rc, st in one["stats"]] == [st.n_chunks for rc, st in grp["stats"]]
    assert_chain_parity(grp, want, REL_TOL_BF16)
    if cap:
        assert sum(st.n_misses for st in stats) > 0


# ---------------------------------------------------------------------------------------------------------------
# arranging window: small groups of missing experts wait for later arrivals; same results, fewer switches, and the
# schedule (who runs in which step, which switches) equals the oracle's replay
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("window", [(0, 6, 3), (3, 8, 2)])
def test_arranging_window_matches_replay_and_keeps_results(B, oracle, G, window):
    from oracle import arrange
    n, E, arrival = 120, 10, 20
    wl = W.config3(n, hw=64, n_experts=E, width=16, cap=4, arrival_batch=arrival, calibrated=False)
    G.calibrate_workload(wl, n_cal=64, targets={0: W.zipf_probs(E - 1, 1.1)})
    blobs = [wl.blob(e) for e in range(E)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    assert not want["ambiguous"].any()
    plain = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=arrival)
    got = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=arrival, arranging=window)
    assert_chain_parity(got, want, REL_TOL_BF16)
    assert np.array_equal(got["path"], plain["path"]) and np.array_equal(got["logits"], plain["logits"])
    # the oracle's replay of the same arrivals, routes from the chain oracle
    sim = oracle.CacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_experts=4)
    log = [(e, []) for e in sim.init_fill()]
    paths = [[int(e) for e in p if e >= 0] for p in want["path"]]
    submits = [list(range(s, min(s + arrival, n))) for s in range(0, n, arrival)]
    rec = arrange.replay(submits, paths, wl.expert_arch, {0: window}, sim)
    stats = [st for rc, st in got["stats"] if rc == B.COE_OK]
    assert len(stats) == len(rec)
    for st, r in zip(stats, rec):
        assert st.n_pending == r["n_pending"] and st.n_groups == len(r["run"]) and st.n_misses == len(r["switches"])
        assert st.n_deferred_groups == len(r["deferred"])
        assert st.n_deferred_requests == sum(len(m) for m in r["deferred"].values())
        log += r["switches"]
    assert got["switch_log"] == log
    assert sum(st.n_deferred_groups for st in stats) > 0
    assert len(got["switch_log"]) < len(plain["switch_log"])         # waiting groups merged: fewer switches
    print(f"window {window}: {len(plain['switch_log']) - 4} -> {len(log) - 4} switches, "
          f"{len([1 for rc, st in plain['stats'] if rc == B.COE_OK])} -> {len(stats)} steps")


def test_offline_profiler_measures_a_usable_latency_model(B):
    """Section 4.5 microbenchmark on a small ResNet-50-shaped architecture: latency grows with the batch, the fitted
    line has a positive slope and intercept, a switch moves exactly the blob, thresholds are ordered."""
    from paper_2503_02354_amd import profiler as P
    arch = W.resnet50(8, 64, W.DT_BF16, 32)
    blob = W.make_expert_blob(arch, 3, 0)
    sizes = [1, 16, 64, 128, 256]
    m = P.profile_arch(arch, blob, sizes, max_batch=256, efficiency=0.2, repeats=5)
    lat = m["latency_us"]
    assert lat[256] > lat[1] and m["K_us"] > 0 and m["B_us"] > 0, m
    assert m["max_batch"] in sizes
    assert m["load_us"] > 0 and 1.0 < m["load_GBps"] < 100.0, m
    assert 0 <= m["min_group_resident"] <= m["min_group_missing"]
    print(f"latency model K {m['K_us']:.2f} us/request, B {m['B_us']:.0f} us, load {m['load_us']:.0f} us at {m['load_GBps']:.1f} GB/s, "
          f"thresholds {m['min_group_resident'], m['min_group_missing']}, max batch {m['max_batch']}")


def test_window_search_on_measured_throughput_with_a_shared_memory_budget(B, oracle, G):
    """Section 4.4 with measured throughputs.  One memory budget is shared by the expert cache and the activation workspace:
    keeping n experts on the device leaves budget - n x blob bytes for activations, which bounds the batch size
    (coe_config.cache_cap_bytes and max_batch are set from the same budget).  Few experts: every group of a missing expert
    costs a switch; many experts: batches shrink.  The search (library arithmetic, throughputs measured here on the GPU) must
    visit the windows the decay rule prescribes and stop for the reason its own trace implies; every configuration it visits
    produces the same routes and logits."""
    from paper_2503_02354_amd import profiler as P
    from oracle import profiler_oracle as PO
    n, E, arrival = 384, 24, 96
    wl = W.config3(n, hw=64, n_experts=E, width=16, cap=0, arrival_batch=arrival, calibrated=False)
    G.calibrate_workload(wl, n_cal=64, targets={0: W.zipf_probs(E - 1, 1.1)})
    blobs = [wl.blob(e) for e in range(E)]
    x = wl.inputs(range(n))
    dev = device_tensor(x)
    blob_bytes = blobs[0].nbytes
    act_per_request = 64 * 64 * 64 * 2 * 6          # a few activation buffers of the largest tensor, per request
    budget = E * blob_bytes + 8 * act_per_request   # with every expert resident only 8 requests fit a batch
    results = {}

    def throughput_at(n_experts):
        cap_bytes = n_experts * blob_bytes
        max_batch = max(1, min(256, (budget - cap_bytes) // act_per_request))
        ctx = B.Context(max_requests=n, max_stages=2, max_batch=int(max_batch), cache_cap_bytes=int(cap_bytes), prefetch_depth=1)
        B.setup_workload(ctx, wl, blobs)
        best = 0.0
        for rep in range(3):
            t0 = time.perf_counter()
            for s in range(0, n, arrival):
                ctx.coe_submit(arrival, dev.data_ptr() + s * x[0].nbytes, True)
                ctx.coe_step()
            while ctx.coe_step()[0] != B.COE_DONE:
                pass
            ids, logits, path = ctx.coe_collect(n)
            best = max(best, n / (time.perf_counter() - t0))
            order = np.argsort(ids)
            results.setdefault("ref", (path[order], logits[order]))
            assert np.array_equal(path[order], results["ref"][0]) and np.array_equal(logits[order], results["ref"][1])
        ctx.close()
        results[n_experts] = (int(max_batch), best)
        return best

    # initial window 6, decay factor 0.94: upper bounds 6, 11.64, 16.94, 21.92, 26.6 -> 6, 12, 17, 22 and all 24 experts
    out = P.search_resident_experts(E, throughput_at, initial_window=6.0, error_margin=0.05, fit_points=2)
    assert out["loaded"] == [6, 12, 17, 22, 24][:len(out["loaded"])] and len(out["loaded"]) >= 3
    # the oracle twin, fed the throughputs measured above, takes the same decisions
    ref = PO.decay_window_search(E, lambda k: results[k][1], 6.0, 0.05, 2)
    assert out["loaded"] == ref["loaded"] and out["experts"] == ref["experts"] and out["stopped_by"] == ref["stopped_by"]
    print("window search on measured throughput:", {k: v for k, v in results.items() if k != "ref"}, out)


@pytest.mark.parametrize("rule,depth", [(1, 0), (2, 0), (0, 1), (0, 2), (1, 2)])
def test_replacement_rules_and_in_use_depth_follow_the_replay(B, oracle, G, rule, depth):
    """Least-recently-used (1) and first-in-first-out (2) replacement in the device cache, and the two-stage rule (0)
    with the experts of the preceding groups protected while a load is in flight: same results as the plain two-stage
    rule, switch log equal to the oracle's replay of that rule."""
    from oracle import arrange
    n, E, arrival = 120, 10, 20
    wl = W.config3(n, hw=64, n_experts=E, width=16, cap=4, arrival_batch=arrival, calibrated=False)
    G.calibrate_workload(wl, n_cal=64, targets={0: W.zipf_probs(E - 1, 1.1)})
    blobs = [wl.blob(e) for e in range(E)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    assert not want["ambiguous"].any()
    base = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=arrival)
    got = run_chain_gpu(B, wl, blobs, x, max_batch=16, arrival=arrival, eviction=rule, prefetch_depth=depth)
    assert np.array_equal(got["path"], base["path"]) and np.array_equal(got["logits"], base["logits"])
    assert_chain_parity(got, want, REL_TOL_BF16)
    sim = oracle.CacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_experts=4, rule=rule,
                          in_use=depth)
    log = [(e, []) for e in sim.init_fill()]
    paths = [[int(e) for e in p if e >= 0] for p in want["path"]]
    submits = [list(range(s, min(s + arrival, n))) for s in range(0, n, arrival)]
    for r in arrange.replay(submits, paths, wl.expert_arch, {}, sim):
        log += r["switches"]
    assert got["switch_log"] == log
    assert got["switch_log"] != base["switch_log"]
    print(f"rule {rule} depth {depth}: {len(log) - 4} switches, plain two-stage rule: {len(base['switch_log']) - 4}")


def test_launch_sequences_respect_the_address_limit(B):
    """Kernels address a tensor with 31-bit byte offsets, so a launch sequence covers at most 2^31 / (largest tensor of
    one request) requests whatever max_batch says.  Here the largest tensor is 256x256x64 bf16 = 8 MiB: 255 requests.
    300 requests with max_batch 4096 must run as two sequences of 150 and give the bits of a run in chunks of 64."""
    p = W._Prog(256, 256, 4)
    p.conv(0, 1, 64, 3, 1, 1, W.ACT_RELU)
    p.head(1, 8)
    arch = W.Arch("wide", W.DT_BF16, 256, 256, 4, 8, np.array(p.layers, dtype=np.int32), p.gains)
    blob = W.make_expert_blob(arch, 5, 0)
    n = 300
    x = W.make_inputs(arch, 5, range(16))
    x = np.concatenate([x] * 19)[:n]                                  # 16 distinct images, repeated
    dev = device_tensor(x)
    outs = []
    for max_batch in (4096, 64):
        ctx = B.Context(max_requests=n, max_stages=1, max_batch=max_batch)
        aid = ctx.coe_register_arch(arch)
        ctx.coe_register_expert(0, aid, blob, 1.0)
        ctx.coe_set_dependency_graph(np.zeros(2, np.int32), np.zeros(0, np.int32))
        ctx.coe_submit(n, dev.data_ptr(), True)
        rc, st = ctx.coe_step()
        assert rc == B.COE_OK and st.n_chunks == (2 if max_batch == 4096 else 5)
        ids, logits, path = ctx.coe_collect(n)
        ctx.close()
        outs.append(logits[np.argsort(ids)])
    assert np.isfinite(outs[0]).all() and np.abs(outs[0]).max() > 0
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(outs[0][:16], outs[0][16:32])               # repeated images, repeated results


def test_steps_allocate_nothing_on_a_capped_two_architecture_dag(B, oracle, G):
    """Expert arena: a cache of 5 of 18 experts of two architectures (two slot classes), so consecutive switches alternate
    between blob sizes.  No step allocates device memory (not even the first), submits of device inputs return without
    waiting, results equal the oracle's and the switch log equals the policy replay's - also with a byte cap that only the
    smaller architecture's slots can use up."""
    n, arrival = 120, 24
    wl = W.config4(n, hw=64, tiers=(3, 6, 9), width=16, fan=(3, 2), calibrated=False)
    G.calibrate_workload(wl, n_cal=32)
    E = wl.graph.n_experts
    blobs = [wl.blob(e) for e in range(E)]
    sizes = sorted(set(b.nbytes for b in blobs))
    assert len(sizes) == 2
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    assert not want["ambiguous"].any()
    for caps in (dict(cache_cap_experts=5), dict(cache_cap_experts=6, cache_cap_bytes=2 * sizes[1] + 3 * sizes[0])):
        ctx = B.Context(max_requests=n, max_stages=wl.max_stages, max_batch=32, prefetch_depth=1, **caps)
        B.setup_workload(ctx, wl, blobs)
        got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, arrival=arrival, ctx=ctx)
        ctx.close()
        assert_chain_parity(got, want, REL_TOL_BF16)
        stats = [st for rc, st in got["stats"] if rc == B.COE_OK]
        assert all(st.n_device_allocs == 0 for st in stats), [st.n_device_allocs for st in stats]
        assert sum(st.n_misses for st in stats) > 10
        sim = oracle.CacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ,
                              cap_experts=caps["cache_cap_experts"], cap_bytes=caps.get("cache_cap_bytes", 0), in_use=1)
        fill = sim.init_fill()
        log = [(e, []) for e in fill]
        keys = np.full(n, -1, np.int64)
        depth = np.zeros(n, np.int64)
        arrived = 0
        for st in stats:
            if arrived < n:
                keys[arrived:arrived + arrival] = want["path"][arrived:arrived + arrival, 0]
                arrived += arrival
            has = np.zeros(E, np.uint8)
            has[keys[keys >= 0]] = 1
            log += sim.stage(has)[1]
            live = keys >= 0
            depth[live] += 1
            nxt = np.full(n, -1, np.int64)
            idx = np.nonzero(live)[0]
            ok = depth[idx] < wl.max_stages
            nxt[idx[ok]] = want["path"][idx[ok], depth[idx[ok]]]
            keys = nxt
        assert got["switch_log"] == log
        sizes_switched = set(blobs[e].nbytes for e, v in log[len(fill):])
        assert sizes_switched == set(sizes)                       # switches of both slot classes happened


def test_arranging_window_on_a_capped_mixed_dag(B, oracle, G):
    """Three-stage DAG with two architectures, requests arriving in five batches, a cache of 7 of the 18 experts, an
    arranging window with different thresholds per architecture and two groups of prefetch: results equal the plain
    schedule's bit for bit and the oracle's within tolerance; which groups run, wait and switch in every step equals
    the oracle's replay."""
    from oracle import arrange
    n, arrival = 150, 30
    wl = W.config4(n, hw=64, tiers=(3, 6, 9), width=16, fan=(3, 2), calibrated=False)
    G.calibrate_workload(wl, n_cal=32)
    E = wl.graph.n_experts
    blobs = [wl.blob(e) for e in range(E)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    assert not want["ambiguous"].any()
    plain = run_chain_gpu(B, wl, blobs, x, wl.first_expert, max_batch=32, arrival=arrival)
    windows = {0: (2, 6, 3), 1: (0, 9, 2)}
    ctx = B.Context(max_requests=n, max_stages=wl.max_stages, max_batch=32, cache_cap_experts=7, prefetch_depth=2)
    B.setup_workload(ctx, wl, blobs)
    for a, w in windows.items():
        ctx.coe_set_arranging(a, *w)
    got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, arrival=arrival, ctx=ctx)
    ctx.close()
    assert np.array_equal(got["path"], plain["path"]) and np.array_equal(got["logits"], plain["logits"])
    assert_chain_parity(got, want, REL_TOL_BF16)
    sim = oracle.CacheSim([b.nbytes for b in blobs], wl.usage_prob, wl.graph.succ_off, wl.graph.succ, cap_experts=7, in_use=2)
    log = [(e, []) for e in sim.init_fill()]
    paths = [[int(e) for e in p if e >= 0] for p in want["path"]]
    submits = [list(range(s, min(s + arrival, n))) for s in range(0, n, arrival)]
    rec = arrange.replay(submits, paths, wl.expert_arch, windows, sim)
    stats = [st for rc, st in got["stats"] if rc == B.COE_OK]
    assert len(stats) == len(rec)
    for st, r in zip(stats, rec):
        assert (st.n_pending, st.n_groups, st.n_misses) == (r["n_pending"], len(r["run"]), len(r["switches"]))
        assert st.n_deferred_groups == len(r["deferred"])
        assert st.n_deferred_requests == sum(len(m) for m in r["deferred"].values())
        log += r["switches"]
    assert got["switch_log"] == log
    assert sum(st.n_deferred_groups for st in stats) > 0 and len(log) > 7


@pytest.mark.parametrize("executors,cap,group_small", [(3, 4, -1), (2, 0, 0), (3, 5, 0)])
def test_executors_give_the_same_bits_and_follow_the_assignment_rule(B, oracle, G, executors, cap, group_small):
    """Several executors (streams with their own activation workspaces): launch sequences of different groups overlap
    on the device.  Same routes and logits bit for bit, same switch log as with one executor; the executor of every
    launch sequence of the last step is what the oracle's assignment rule gives for the library's predicted costs, and
    those costs are K n + B (+ load for a missing expert) where a launch sequence is one group."""
    from oracle import arrange
    n, E, arrival = 160, 16, 40
    wl = W.config2(n, hw=64, n_experts=E, width=64, calibrated=False)
    G.calibrate_workload(wl, n_cal=48)
    blobs = [wl.blob(e) for e in range(E)]
    x, sub, want, _ = G.guarded_inputs(wl, blobs, range(n))
    lat = (700, 90000, 50000)
    one = run_chain_gpu(B, wl, blobs, x, max_batch=64, arrival=arrival, cap_experts=cap, group_small=group_small, latency=lat)
    got = run_chain_gpu(B, wl, blobs, x, max_batch=64, arrival=arrival, cap_experts=cap, group_small=group_small, latency=lat,
                        executors=executors, keep=True)
    ctx = got.pop("ctx")
    assert np.array_equal(one["path"], got["path"]) and np.array_equal(one["logits"], got["logits"])
    assert one["switch_log"] == got["switch_log"]
    assert_chain_parity(got, want, REL_TOL_BF16)
    assert max(st.n_executors_used for rc, st in got["stats"]) == executors
    assert all(st.n_executors_used == 1 for rc, st in one["stats"] if rc == B.COE_OK and st.n_groups)
    fe, cost, ex = ctx.coe_debug_last_assignment()
    ctx.close()
    assert len(fe) >= 1 and ex.tolist() == arrange.assign(cost.tolist(), executors)
    if group_small < 0:                                  # one launch sequence per group: the cost model is checkable
        last = [st for rc, st in got["stats"] if rc == B.COE_OK][-1]
        sizes = np.bincount(want["path"][n - arrival:, 1], minlength=E)          # the last step runs the last arrival's leaves
        misses = {e for e, v in got["switch_log"][-last.n_misses:]} if last.n_misses else set()
        for e, cst in zip(fe.tolist(), cost.tolist()):
            assert cst == lat[0] * int(sizes[e]) + lat[1] + (lat[2] if e in misses else 0), (e, cst)
