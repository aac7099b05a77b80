"""GPU parity of the LAMB step against the oracle, through the C ABI.  All arithmetic is fp32 on the GPU: master
weights, moments and trust ratio within 1e-5 (max-normalised); the bf16 copy of the weights within one bf16 unit."""
import numpy as np
import pytest
import torch

from oracle.lamb import lamb_step
from stage_util import max_norm_err

pytestmark = pytest.mark.gpu


def _run(n, steps, seed, param_dtype=torch.bfloat16, **hyper):
    import paper_2301_11913_amd as sw
    rng = np.random.default_rng(seed)
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(steps)]
    wd, md, vd = torch.from_numpy(w0.copy()).cuda(), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    pd = torch.zeros(n, dtype=param_dtype, device="cuda") if param_dtype is not None else None
    ws = torch.empty(sw.swarm_lamb_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ratio = torch.zeros(1, device="cuda")
    w, m, v = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, start=1):
        sw.swarm_lamb_step(wd, pd, torch.from_numpy(g).cuda(), md, vd, t, ws, trust_ratio=ratio, **hyper)
        torch.cuda.synchronize()
        w, m, v, r = lamb_step(w, g, m, v, t, **hyper)
        assert abs(ratio.item() - r) <= 1e-5 * r, (t, ratio.item(), r)
        assert max_norm_err(wd.cpu().numpy(), w) <= 1e-5, t
        assert max_norm_err(md.cpu().numpy(), m) <= 1e-5 and max_norm_err(vd.cpu().numpy(), v) <= 1e-5, t
        if pd is not None:
            got = pd.float().cpu().numpy().astype(np.float64)
            unit = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(w), 1e-30))) - (7 if param_dtype == torch.bfloat16 else 23))
            assert np.all(np.abs(got - w) <= unit + 1e-9), t
            assert torch.equal(pd, wd.to(param_dtype))          # the copy is the rounded master weight, exactly
    return wd


@pytest.mark.parametrize("n", [1, 7, 4096, 4099, 1 << 20, (1 << 20) + 13])
def test_lamb_steps(n):
    _run(n, 3, seed=n % 97)


def test_lamb_hyperparameters_and_fp32_copy():
    _run(50000, 2, seed=5, param_dtype=torch.float32, lr=2e-3, beta1=0.8, beta2=0.99, eps=1e-8, weight_decay=0.0,
         grad_scale=0.25)
    _run(50000, 2, seed=6, param_dtype=None, weight_decay=0.1)


def test_lamb_zero_gradient_and_zero_weights():
    import paper_2301_11913_amd as sw
    n = 3000
    ws = torch.empty(sw.swarm_lamb_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    w = torch.full((n,), 0.5, device="cuda"); z = lambda: torch.zeros(n, device="cuda")
    ratio = torch.zeros(1, device="cuda")
    sw.swarm_lamb_step(w, None, z(), z(), z(), 1, ws, lr=1e-3, weight_decay=0.01, trust_ratio=ratio)
    torch.cuda.synchronize()
    assert abs(ratio.item() - 100.0) < 1e-3 and torch.allclose(w, torch.full_like(w, 0.5 * (1 - 1e-3)), rtol=1e-6)
    w0 = z()
    sw.swarm_lamb_step(w0, None, torch.full((n,), 2.0, device="cuda"), z(), z(), 1, ws, lr=1e-3, eps=1e-6, trust_ratio=ratio)
    torch.cuda.synchronize()
    assert ratio.item() == 1.0 and torch.allclose(w0, torch.full_like(w0, -1e-3), rtol=1e-5)


def test_lamb_is_reproducible():
    a = _run(300001, 2, seed=9)
    b = _run(300001, 2, seed=9)
    assert torch.equal(a, b)


@pytest.mark.timeout(600)
def test_lamb_largest_tensor_of_the_bench_workload():
    """The launch configuration bench.py times: w_1 of the Section 4.3 stage (134 M elements), two steps, every
    element against the oracle."""
    import swarm_synth as synth
    import paper_2301_11913_amd as sw
    wl = synth.LAMB_WORKLOADS["lamb_stage_rope_geglu_d4096"]
    big = max(range(len(wl.shapes)), key=lambda i: int(np.prod(wl.shapes[i])))
    w0, g = synth.make_lamb_tensor(wl, big)
    n = w0.size
    assert n == 32768 * 4096
    wd, gd = torch.from_numpy(w0).cuda(), torch.from_numpy(g).cuda()
    md, vd = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    pd = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(sw.swarm_lamb_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ratio = torch.zeros(1, device="cuda")
    w, m, v = w0, np.zeros(n), np.zeros(n)
    for t in (1, 2):
        sw.swarm_lamb_step(wd, pd, gd, md, vd, t, ws, trust_ratio=ratio)
        torch.cuda.synchronize()
        w, m, v, r = lamb_step(w, g, m, v, t)
        assert abs(ratio.item() - r) <= 1e-5 * r
        for got, ref in ((wd, w), (md, m), (vd, v)):
            d = np.abs(got.cpu().numpy().astype(np.float64) - ref).max()
            assert d <= 1e-5 * np.abs(ref).max(), t
        assert torch.equal(pd, wd.to(torch.bfloat16))
