"""swarm_lamb_step_static (the LAMB step for callers that cannot allocate: its scratch is a static device array in
the library) against swarm_lamb_step, bit for bit, through the C ABI: two calls in a row on the shared scratch,
the second on a smaller tensor, then the size limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _state(n, seed):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    v = (rng.random(n) * 1e-6).astype(np.float32)
    return w, g, m, v


def _both(n, seed, step):
    import paper_2301_11913_amd as sw
    w, g, m, v = _state(n, seed)
    out = []
    for static in (False, True):
        wd, gd, md, vd = (torch.from_numpy(a.copy()).cuda() for a in (w, g, m, v))
        pd = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
        ratio = torch.zeros(1, device="cuda")
        if static:
            sw.swarm_lamb_step_static(wd, pd, gd, md, vd, step, trust_ratio=ratio)
        else:
            ws = torch.empty(sw.swarm_lamb_workspace_bytes(n), dtype=torch.uint8, device="cuda")
            sw.swarm_lamb_step(wd, pd, gd, md, vd, step, ws, trust_ratio=ratio)
        torch.cuda.synchronize()
        out.append((wd, pd, md, vd, ratio))
    for a, b in zip(*out):
        assert torch.equal(a, b)
    assert not torch.equal(out[1][0], torch.from_numpy(w).cuda())     # the update did happen


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    _both((1 << 22) + 4099, seed=1, step=1)      # several hundred workgroups and a ragged tail
    _both(70001, seed=2, step=3)                 # smaller tensor on the scratch the first call left behind
    _both(5, seed=3, step=2)


def test_static_scratch_largest_size_and_limit():
    import paper_2301_11913_amd as sw
    n = sw.SWARM_LAMB_STATIC_MAX_ELEMS
    _both(n, seed=4, step=1)
    big = torch.zeros(n + 1, device="cuda")
    with pytest.raises(sw.SwarmError) as e:
        sw.swarm_lamb_step_static(big, None, big, big, big, 1)
    assert e.value.status == -4                   # SWARM_ERR_WORKSPACE, before any launch
