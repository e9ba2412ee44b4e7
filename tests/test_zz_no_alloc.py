"""The entry point that allocates nothing (coe_regroup_static: histogram scratch in a static device array) against the
existing stand-alone regroup entry point (coe_debug_regroup, scratch owned by a context), bit for bit, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, so that stale scratch contents of the first call
would show."""
import numpy as np
import pytest



def _static_regroup(B, torch, keys, n_experts):
    n = len(keys)
    cur = torch.from_numpy(keys).cuda()
    # outputs start as garbage: everything the contract defines must be overwritten
    cnt = torch.full((n_experts,), -7, dtype=torch.int32, device="cuda")
    off = torch.full((n_experts + 1,), -7, dtype=torch.int32, device="cuda")
    perm = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
    inv = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream
    B.coe_regroup_static(n, cur.data_ptr(), n_experts, cnt.data_ptr(), off.data_ptr(), perm.data_ptr(), inv.data_ptr(), stream)
    torch.cuda.synchronize()
    off_h = off.cpu().numpy()
    m = int(off_h[n_experts])
    return dict(n_pending=m, cnt=cnt.cpu().numpy(), off=off_h, perm=perm.cpu().numpy()[:m], inv=inv.cpu().numpy()[:n])


@pytest.mark.gpu
def test_static_scratch_regroup_matches_the_context_one_twice_in_a_row():
    import torch
    assert torch.cuda.is_available()
    from paper_2503_02354_amd import binding as B
    rng = np.random.default_rng(7)
    # (requests, experts): several workgroups with a ragged tail and finished requests (-1) in between, then a smaller
    # input with other keys and fewer experts, then the largest shape the scratch takes
    cases = [(16384 + 37, 120), (1000, 64), (5, 3), (256 * 512, 2048)]
    ctx = B.Context(max_requests=max(n for n, _ in cases))
    try:
        for n, E in cases:
            keys = rng.integers(-1, E, size=n).astype(np.int32)
            keys[rng.random(n) < 0.05] = E + 3            # out-of-range ids count as not queued
            want = ctx.coe_debug_regroup(keys, E)
            got = _static_regroup(B, torch, keys, E)
            assert got["n_pending"] == want["n_pending"], (n, E)
            for k in ("cnt", "off", "perm", "inv"):
                assert np.array_equal(got[k], want[k]), (n, E, k)
    finally:
        ctx.close()


def test_static_scratch_regroup_rejects_what_does_not_fit():
    """Sizes are checked before anything touches a device: no GPU needed (the pointers are never followed)."""
    import pytest
    from paper_2503_02354_amd import binding as B
    t = np.zeros(8, np.int32)
    a = t.ctypes.data
    with pytest.raises(B.CoEError) as e:
        B.coe_regroup_static(256 * 513, a, 2048, a, a, a, a, 0)
    assert e.value.code == B.COE_ERANGE and "exceeds the static scratch" in str(e.value)
    with pytest.raises(B.CoEError) as e:
        B.coe_regroup_static(8, a, 4096, a, a, a, a, 0)
    assert e.value.code == B.COE_EINVAL
    with pytest.raises(B.CoEError) as e:
        B.coe_regroup_static(8, a, 4, 0, a, a, a, 0)
    assert e.value.code == B.COE_EINVAL
