"""The stage entry points launch kernels on the caller's stream and nothing else (no allocation, no memset, no
synchronisation), so a caller may record them into a HIP graph.  A recorded step is replayed several times, with
eager work of the same library and synchronisations between the replays, and every replay must reproduce the eager
results bit for bit (the gradients are added to, so each replay starts from cleared sums)."""
import pytest
import torch

import swarm_synth as synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", [
    # dtype, d, H, f, S, B, L, R, coded
    ("bf16", 256, 2, 512, 160, 2, 1, 2, True),       # shared block: the one device-to-device copy is recorded too
    ("bf16", 512, 4, 1024, 75, 3, 2, 1, True),
    ("f32", 256, 4, 1024, 64, 2, 1, 1, False),
])
def test_stage_step_replays_from_a_graph(case):
    import paper_2301_11913_amd as sw
    dtype, d, H, f, S, B, L, R, coded = case
    wl = synth.Workload(name="graph", dtype=dtype, d_model=d, n_heads=H, d_ffn=f, seq=S, batch=B, n_layers=L,
                        n_repeat=R, grad_sigma=1.0 if dtype == "f32" else 1e-2, seed=31 + d + S)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(a).to(dt).cuda()
    params = [{k: dev(p[k]) for k in sw.PARAM_FIELDS} for p in synth.make_params(wl)]
    x_src, g_src = dev(synth.make_x_in(wl)), dev(synth.make_grad_out(wl))
    cfg = sw.StageConfig(wl.d_model, wl.n_heads, wl.d_ffn, wl.n_layers, wl.n_repeat, wl.batch, wl.seq, wl.dtype,
                         block_kind=wl.block)
    n = x_src.numel()
    grads = [{k: torch.zeros(p[k].shape, dtype=torch.float32, device="cuda") for k in sw.PARAM_FIELDS} for p in params]
    if coded:
        ws = torch.empty(max(sw.swarm_stage_coded_workspace_bytes(cfg, True), sw.swarm_stage_coded_workspace_bytes(cfg, False)),
                         dtype=torch.uint8, device="cuda")
        c = {k: torch.empty(n, dtype=torch.int8, device="cuda") for k in ("x", "g", "y", "gin")}
        s = {k: torch.empty(n // 64, dtype=torch.float32, device="cuda") for k in ("x", "g", "y", "gin")}
        sw.swarm_codec_encode(x_src, c["x"], s["x"])
        sw.swarm_codec_encode(g_src, c["g"], s["g"])
        xdec = torch.empty_like(x_src)
        outs = [c["y"], s["y"], c["gin"], s["gin"], xdec]

        def step():
            sw.swarm_stage_forward_coded(cfg, params, c["x"], s["x"], xdec, c["y"], s["y"], ws)
            sw.swarm_stage_backward_coded(cfg, params, xdec, c["g"], s["g"], c["gin"], s["gin"], grads, ws)
    else:
        ws = torch.empty(sw.swarm_stage_workspace_bytes(cfg, True), dtype=torch.uint8, device="cuda")
        y, gin = torch.empty_like(x_src), torch.empty_like(x_src)
        outs = [y, gin]

        def step():
            sw.swarm_stage_forward(cfg, params, x_src, y, ws)
            sw.swarm_stage_backward(cfg, params, x_src, g_src, gin, grads, ws)

    all_out = lambda: outs + [g[k] for g in grads for k in sw.PARAM_FIELDS]

    def clear():
        for g in grads:
            for k in g:
                g[k].zero_()
        for o in outs:
            o.fill_(3)

    clear()
    step()                                   # eager: also the first call on this device (opt-ins happen here)
    torch.cuda.synchronize()
    want = [t.clone() for t in all_out()]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()

    for i in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(all_out(), want):
            assert torch.equal(got, ref), "replay %d" % i
        # eager work of the library and a synchronisation between the replays
        clear()
        step()
        torch.cuda.synchronize()
        for got, ref in zip(all_out(), want):
            assert torch.equal(got, ref), "eager after replay %d" % i
