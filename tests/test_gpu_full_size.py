"""Full-size configurations on the GPU in the launch configuration bench.py times.  The oracle cannot run every
request at these sizes, so: a seeded sample of requests (margin-guarded, re-drawn where needed) is compared with the
oracle one by one; every request is checked through properties that hold at any size (valid path through the graph,
regroup = stable sort of the routed ids, identical results when the sampled requests run alone)."""
import numpy as np
import pytest

from paper_2503_02354_amd import workloads as W

pytestmark = pytest.mark.gpu

from gpu_util import REL_TOL_BF16, device_tensor, rel_err, run_chain_gpu  # noqa: E402


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2503_02354_amd import binding
    return binding


def _valid_paths(path, wl):
    for r, p in enumerate(path):
        p = [int(v) for v in p if v >= 0]
        assert p and p[0] == (0 if wl.first_expert is None else int(wl.first_expert[r]))
        for a, b in zip(p, p[1:]):
            assert b in wl.graph.successors(a).tolist()
        succ = wl.graph.successors(p[-1]).tolist()
        assert len(succ) == 0 or -1 in succ, "request stopped at an expert that still routes"


def _sampled_case(B, oracle, wl, n_sample, max_batch, arrival=None, seed=1):
    from oracle import guard as G
    n = wl.n_requests
    E = wl.graph.n_experts
    blobs = [wl.blob(e) for e in range(E)]
    rng = np.random.default_rng(seed)
    sample = np.sort(rng.choice(n, size=n_sample, replace=False))
    xs, sub, want, redraws = G.guarded_inputs(wl, blobs, sample)
    subseeds = np.zeros(n, np.int32)
    subseeds[sample] = sub
    x = wl.inputs(range(n), subseeds)
    assert np.array_equal(x[sample], xs)
    got = run_chain_gpu(B, wl, blobs, x, wl.first_expert, max_batch=max_batch, arrival=arrival, keep=True)
    ctx = got.pop("ctx")
    # sampled requests against the oracle
    assert np.array_equal(got["path"][sample], want["path"]), "routes of sampled requests differ from the oracle"
    err = rel_err(got["logits"][sample][:, :want["logits"].shape[1]], want["logits"])
    assert err.max() <= REL_TOL_BF16, err.max()
    # every request: valid path
    _valid_paths(got["path"], wl)
    # the sampled requests alone give the same bits: results do not depend on grouping or batch composition
    alone = run_chain_gpu(B, wl, blobs, xs, None if wl.first_expert is None else wl.first_expert[sample], max_batch=max_batch)
    assert np.array_equal(alone["path"], got["path"][sample])
    assert np.array_equal(alone["logits"], got["logits"][sample])
    ctx.close()
    return got, want, sample, float(err.max()), redraws


def test_config2_full_size(B, oracle):
    """16 ResNet-18-shaped bf16 experts, 4096 requests of 3x224x224, root routes 15 ways, all resident."""
    wl = W.config2()
    assert wl.head_bias, "calibration file missing"
    got, want, sample, err, redraws = _sampled_case(B, oracle, wl, n_sample=48, max_batch=512)
    # the regroup of the second stage is the stable sort of the routed ids (all 4096 requests, bit exact):
    # replay stage 2's keys through the library's regroup and the oracle's
    keys = got["path"][:, 1].astype(np.int32)
    ctx = B.Context(max_requests=wl.n_requests)
    dev = ctx.coe_debug_regroup(keys, wl.graph.n_experts)
    ctx.close()
    ref = oracle.regroup(keys, wl.graph.n_experts)
    for k in ("cnt", "off", "perm", "inv"):
        assert np.array_equal(dev[k], ref[k]), k
    assert [st.n_groups for rc, st in got["stats"][:2]] == [1, int((ref["cnt"] > 0).sum())]
    leaves = ref["cnt"][1:]
    assert leaves.min() > 100 and leaves.max() < 600, leaves          # calibration spreads the 15 routes
    print(f"config2 full size: {len(sample)} sampled requests, max rel err {err:.2e}, {redraws} re-draws, leaves {leaves.tolist()}")
