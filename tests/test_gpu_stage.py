"""GPU parity of the stage forward/backward against the oracle, through the C ABI.

Tolerances (benchmark description): fp32 within 1e-4, bf16 within 2e-2, both as
max|gpu - oracle| / max|oracle| per output tensor (x_out, grad_in, every grad_params field).
The oracle runs in fp64 on the same (bf16-rounded where applicable) inputs.
"""
import numpy as np
import pytest
import torch

import swarm_synth as synth
from stage_util import run_gpu, run_oracle, compare

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _check(wl, **kw):
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    gpu = run_gpu(wl, params, x, G, **kw)
    ref = run_oracle(wl, params, x, G, **kw)
    errs, bad = compare(gpu, ref, TOL[wl.dtype])
    print(wl.name, {k: "%.2e" % v for k, v in errs.items()})
    assert not bad, bad
    return gpu, ref


def test_config1_block_f32():
    _check(synth.WORKLOADS["block_f32_d256"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    # d, H, f, S, B, L, R : ragged token counts, several tiles, both head sizes, sharing
    (128, 2, 192, 37, 3, 1, 1),
    (256, 2, 320, 150, 2, 2, 1),
    (128, 1, 256, 65, 1, 1, 3),
    (192, 3, 448, 1, 5, 2, 2),
])
def test_small_ragged(dtype, shape):
    d, H, f, S, B, L, R = shape
    wl = synth.Workload(name="ragged", dtype=dtype, d_model=d, n_heads=H, d_ffn=f, seq=S, batch=B, n_layers=L,
                        n_repeat=R, grad_sigma=1.0 if dtype == "f32" else 1e-2, seed=4242 + d + S)
    _check(wl)


@pytest.mark.parametrize("case", [
    # dtype, d_model, heads: widths whose 8-element chunks do not fill the last pass of the LayerNorm kernels' lanes
    # (768, 1536, 6144) and the widest model the stage accepts (8192), few tokens
    ("bf16", 768, 6), ("f32", 768, 12), ("bf16", 1536, 12), ("f32", 1536, 24), ("bf16", 6144, 48), ("f32", 6144, 48),
    ("bf16", 8192, 64),
])
def test_wide_models(case):
    dtype, d, H = case
    wl = synth.Workload(name="wide", dtype=dtype, d_model=d, n_heads=H, d_ffn=1024 if d > 2048 else 2 * d, seq=40, batch=2,
                        n_layers=1, n_repeat=1, grad_sigma=1.0 if dtype == "f32" else 1e-2, seed=99 + d)
    _check(wl)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_rows(dtype):
    """Token rows the LayerNorm has nothing to normalise (all features equal: variance 0, the row statistics rest on
    eps alone), an all-zero row and an all-zero gradient row, next to ordinary ones.  bf16 takes the zero rows only: a
    constant row of -3 makes the hidden stream -3 + (attention output of a few hundredths), which bf16 storage
    quantises to two or three levels before the second LayerNorm divides by their spread; the fp64 oracle keeps
    those digits, and the difference (7 % on the weight gradients) is the storage format's, not a kernel's."""
    wl = synth.Workload(name="degenerate", dtype=dtype, d_model=256, n_heads=2, d_ffn=512, seq=24, batch=2, n_layers=2,
                        n_repeat=1, grad_sigma=1.0 if dtype == "f32" else 1e-2, seed=5)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl).copy(), synth.make_grad_out(wl).copy()
    if dtype == "f32":
        x[0, 3, :] = 0.75
        x[1, 7, :] = -3.0
    x[1, 0, :] = 0.0
    G[0, 5, :] = 0.0
    gpu = run_gpu(wl, params, x, G)
    ref = run_oracle(wl, params, x, G)
    errs, bad = compare(gpu, ref, TOL[wl.dtype])
    assert not bad, bad
    assert np.all(np.isfinite(gpu["x_out"])) and np.all(np.isfinite(gpu["grad_in"]))


def test_config2_stage_bf16():
    _check(synth.WORKLOADS["stage2_bf16_d1024"])


def test_accumulation_and_determinism():
    """grad_params are added to: two backward calls give exactly twice one call's fp32 sums (bitwise, since
    x + x is exact), and repeated calls are bitwise reproducible."""
    wl = synth.WORKLOADS["block_f32_d256"].replace(seq=64, batch=2)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    one = run_gpu(wl, params, x, G, forward=False)
    two = run_gpu(wl, params, x, G, n_backward_calls=2, forward=False)
    again = run_gpu(wl, params, x, G, forward=False)
    for k in one["grads"][0]:
        assert np.array_equal(one["grads"][0][k], again["grads"][0][k]), k
        assert np.array_equal(2.0 * one["grads"][0][k], two["grads"][0][k]), k
    assert np.array_equal(one["grad_in"], again["grad_in"])


def test_forward_and_backward_replay_from_a_hip_graph():
    """The entry points only enqueue kernels and one device-to-device copy on the given stream (no allocation, no
    memset, no synchronisation), so a captured forward + backward replays: three replays, each after eager work
    that dirties the outputs, give bitwise the eager results; grad_params grow by one contribution per replay."""
    import paper_2301_11913_amd as sw
    from stage_util import to_dev
    wl = synth.WORKLOADS["stage2_bf16_d1024"].replace(seq=128, batch=2)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    cfg = sw.StageConfig(wl.d_model, wl.n_heads, wl.d_ffn, wl.n_layers, wl.n_repeat, wl.batch, wl.seq, wl.dtype,
                         wl.ln_eps, wl.block)
    dp = [{k: to_dev(p[k], wl) for k in sw.PARAM_FIELDS} for p in params]
    xd, Gd = to_dev(x, wl), to_dev(G, wl)
    ws_f = torch.empty(sw.swarm_stage_workspace_bytes(cfg, False), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(sw.swarm_stage_workspace_bytes(cfg, True), dtype=torch.uint8, device="cuda")
    new_grads = lambda: [{k: torch.zeros(p[k].shape, dtype=torch.float32, device="cuda") for k in sw.PARAM_FIELDS}
                         for p in params]
    # eager reference (also the warm-up that opts the kernels into their LDS sizes before the capture)
    y0, gin0, gp0 = torch.empty_like(xd), torch.empty_like(xd), new_grads()
    sw.swarm_stage_forward(cfg, dp, xd, y0, ws_f)
    sw.swarm_stage_backward(cfg, dp, xd, Gd, gin0, gp0, ws_b)
    torch.cuda.synchronize()
    y, gin, gp = torch.empty_like(xd), torch.empty_like(xd), new_grads()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sw.swarm_stage_forward(cfg, dp, xd, y, ws_f)
        sw.swarm_stage_backward(cfg, dp, xd, Gd, gin, gp, ws_b)
    for g in gp:                      # whatever the capture itself did to the accumulators is discarded
        for t in g.values():
            t.zero_()
    for n in range(1, 4):
        y.fill_(3.0); gin.fill_(3.0); ws_f.fill_(0xA5); ws_b.fill_(0x5A)   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y0) and torch.equal(gin, gin0), n
        for g, g0 in zip(gp, gp0):
            for k in g:
                one = g0[k].double()
                assert torch.allclose(g[k].double(), n * one, rtol=1e-6, atol=1e-6 * float(one.abs().max())), (n, k)


def test_shared_equals_unrolled_on_gpu():
    wl = synth.Workload(name="shared", dtype="bf16", d_model=256, n_heads=2, d_ffn=512, seq=96, batch=2,
                        n_layers=1, n_repeat=3, grad_sigma=1e-2, seed=77)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    shared = run_gpu(wl, params, x, G)
    unrolled = run_gpu(wl.replace(n_layers=3, n_repeat=1), [params[0]] * 3, x, G)
    assert np.array_equal(shared["x_out"], unrolled["x_out"])
    assert np.array_equal(shared["grad_in"], unrolled["grad_in"])
    for k in shared["grads"][0]:
        tot = sum(unrolled["grads"][l][k] for l in range(3))
        den = np.max(np.abs(tot)) or 1.0
        assert np.max(np.abs(shared["grads"][0][k] - tot)) / den < 1e-5, k


def test_argument_validation_on_device():
    import paper_2301_11913_amd as sw
    wl = synth.WORKLOADS["block_f32_d256"].replace(seq=8, batch=1)
    cfg = sw.StageConfig(wl.d_model, wl.n_heads, wl.d_ffn, 1, 1, wl.batch, wl.seq, wl.dtype)
    params = [{k: torch.zeros(s, device="cuda") for k, s in wl.param_shapes().items()}]
    x = torch.zeros(1, 8, 256, device="cuda")
    y = torch.full_like(x, 5.0)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sw.SwarmError) as e:
        sw.swarm_stage_forward(cfg, params, x, y, small)
    assert e.value.status == -4
    torch.cuda.synchronize()
    assert torch.all(y == 5.0)          # outputs untouched on a host-detected error
