"""Helpers of the GPU parity tests: drive the library through its binding, compare with the oracle."""
import numpy as np

REL_TOL_BF16 = 2e-2    # bf16 in, fp32 accumulate: max |g - o| over classes / max |o| over classes, per request
REL_TOL_F32 = 1e-4     # fp32 experts: only the summation order differs (fp32 FMA chain vs fp64)


def device_tensor(x: np.ndarray):
    """Upload a numpy array (uint16 = bf16 bits, or float32); returns a torch tensor kept alive by the caller."""
    import torch
    t = torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x)
    return t.cuda()


def run_chain_gpu(B, wl, blobs, x, first_expert=None, *, max_batch=0, cap_experts=None, arrival=None, on_device=True,
                  profile=False, ctx=None, keep=False, group_small=0, arranging=None, eviction=0, prefetch_depth=0, executors=0, latency=None,
                  host_tier=None):
    """Submit x in arrival batches, one coe_step after each submit, then step until done; collect everything.
    arranging: (min_group_resident, min_group_missing, max_wait_steps) set for every architecture.
    host_tier: (host_cap_experts, backing_path): experts live in that file, at most so many of them in pinned host memory.
    Returns dict(logits, path, ids, stats, switch_log, host_log[, ctx])."""
    import torch
    n = x.shape[0]
    own = ctx is None
    if own:
        ctx = B.Context(max_requests=max(n, 1), max_stages=wl.max_stages, max_batch=max_batch,
                        cache_cap_experts=wl.cache_cap_experts if cap_experts is None else cap_experts, profile=profile,
                        group_small=group_small, eviction=eviction, prefetch_depth=prefetch_depth, executors=executors)
        if host_tier is not None:
            ctx.coe_set_host_tier(*host_tier)
        B.setup_workload(ctx, wl, blobs)
    if arranging is not None:
        for a in range(len(wl.archs)):
            ctx.coe_set_arranging(a, *arranging)
    if latency is not None:                    # (k_ns, b_ns, load_ns) for every architecture
        for a in range(len(wl.archs)):
            ctx.coe_set_latency_model(a, *latency)
    arrival = arrival or n or 1
    stats = []
    dev = device_tensor(x) if on_device and n else None
    per = x[0].nbytes if n else 0
    for s in range(0, n, arrival):
        m = min(arrival, n - s)
        fe = None if first_expert is None else first_expert[s:s + m]
        if on_device:
            ctx.coe_submit(m, dev.data_ptr() + s * per, True, fe)
        else:
            ctx.coe_submit(m, x[s:s + m], False, fe)
        rc, st = ctx.coe_step()
        stats.append((rc, st))
    for _ in range(64):
        rc, st = ctx.coe_step()
        stats.append((rc, st))
        if rc == B.COE_DONE:
            break
    else:
        raise AssertionError("chain did not finish")
    ids, logits, path = ctx.coe_collect(max(n, 1))
    order = np.argsort(ids)
    out = dict(ids=ids[order], logits=logits[order], path=path[order], stats=stats, switch_log=ctx.coe_debug_switch_log(),
               host_log=ctx.coe_debug_host_log())
    if keep:
        out["ctx"] = ctx
    elif own:
        ctx.close()
    torch.cuda.synchronize()
    return out


def rel_err(g: np.ndarray, o: np.ndarray) -> np.ndarray:
    """Per request: max_c |g_c - o_c| / max(max_c |o_c|, 1e-6)."""
    return np.abs(g.astype(np.float64) - o.astype(np.float64)).max(axis=1) / np.maximum(np.abs(o).max(axis=1), 1e-6)


def assert_chain_parity(got, want, tol, admissible=None):
    """Routes bit-exact and logits within tol.  Requests the margin guard left ambiguous (want["ambiguous"]) must
    instead equal one of the outcomes admissible(i) enumerates: a list of (path, logits) from the oracle alone."""
    amb = want.get("ambiguous")
    amb = np.zeros(len(want["path"]), bool) if amb is None else amb
    clear = ~amb
    bad = np.nonzero((got["path"] != want["path"]).any(axis=1) & clear)[0]
    assert len(bad) == 0, f"route mismatch on requests {bad[:10]}"
    ncls = want["logits"].shape[1]
    err = rel_err(got["logits"][:, :ncls], want["logits"])
    worst = float(err[clear].max()) if clear.any() else 0.0
    assert worst <= tol, f"logit error {worst:.3e} > {tol}"
    for i in np.nonzero(amb)[0]:
        assert admissible is not None, "ambiguous requests need the admissible-outcome enumerator"
        ok = False
        for path, lg in admissible(int(i)):
            if np.array_equal(path, got["path"][i]):
                e = rel_err(got["logits"][i:i + 1, :ncls], lg[None, :ncls])[0]
                worst = max(worst, float(e))
                ok = e <= tol
                break
        assert ok, f"request {i}: route {got['path'][i]} is not an admissible outcome or its logits are off"
    return worst
