#!/usr/bin/env python3
"""Benchmark of the SWARM pipeline-stage hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = what a stage peer does for one microbatch: decode the int8 stage input and the int8
output gradient, stage forward, checkpoint-recomputing stage backward (parameter gradients
accumulated), encode the stage output and the input gradient.  Inputs are synthetic and already
resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E


def measured_traffic(workload, kernel="gemm_bf16"):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (None if there is none)."""
    path = os.path.join(ROOT, "profiles", "%s_%s_hbm_traffic.json" % (kernel, workload))
    try:
        with open(path) as f:
            return json.load(f)["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def attainable_peak():
    """TFLOP/s that a loop of nothing but MFMAs on random bf16 operands sustains on this chip (committed
    micro-benchmark summary; None if there is none): the ceiling the power budget leaves under the nominal peak."""
    try:
        with open(os.path.join(ROOT, "profiles", "mfma_rate_microbench.json")) as f:
            return float(json.load(f)["attainable_tflops_random_16x16x32"])
    except (OSError, KeyError, ValueError):
        return None


EPI_NAMES = {0: "store", 1: "bias", 2: "bias+residual", 3: "bias+gelu", 4: "x gelu'", 5: "fp32 +=", 6: "bias+residual->int8",
             7: "bias+rotary", 8: "x geglu'", 9: "bias+geglu"}


def timed_steps(step, steps, warmup):
    """W warm-up steps, then exactly K steps between two synchronisations (mean from the host clock) with an event
    pair round every step on the launch stream (median and min)."""
    import torch
    for _ in range(warmup):
        step()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    mean_ms = (time.perf_counter() - t0) * 1e3 / steps
    per = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    return mean_ms, per[len(per) // 2], per[0]


def gemm_roofline(step, steps, ms_per_step, workload):
    """Roofline of the dominant kernel (the bf16 MFMA GEMM): the same step run through the instrumented build of the
    library, whose GEMM dispatcher records an event pair on the launch stream round every GEMM launch."""
    import paper_2301_11913_amd as sw
    with sw.using_hooks_library() as lib:
        lib.swarm_kernel_timing_enable.restype = C.c_int
        lib.swarm_kernel_timing_collect_launches.restype = C.c_int
        lib.swarm_kernel_timing_collect_launches.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double),
                                                             C.POINTER(C.c_double), C.POINTER(C.c_int), C.c_int]
        step()                                             # first call through this build (sets LDS sizes)
        import torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(min(steps, 5)):
            step()
        torch.cuda.synchronize()
        ms_hooks = (time.perf_counter() - t0) * 1e3 / min(steps, 5)
        room = 8192
        per_ms, shapes = (C.c_double * room)(), (C.c_int * (6 * room))()
        tot_ms, tot_fl, launches, by_shape = 0.0, 0.0, 0, {}
        for _ in range(steps):
            lib.swarm_kernel_timing_enable(1)
            step()
            ms, fl = C.c_double(), C.c_double()
            nl = lib.swarm_kernel_timing_collect_launches(C.byref(ms), C.byref(fl), per_ms, shapes, room)
            tot_ms += ms.value; tot_fl += fl.value; launches += nl
            for i in range(min(nl, room)):
                key = tuple(shapes[6 * i:6 * i + 6])
                e = by_shape.setdefault(key, [0, 0.0])
                e[0] += 1; e[1] += per_ms[i]
        lib.swarm_kernel_timing_enable(0)
    achieved = tot_fl / (tot_ms * 1e-3) / 1e12
    table = []
    for (M, N, K, at, bt, epi), (cnt, ms) in sorted(by_shape.items(), key=lambda kv: -kv[1][1]):
        tf = 2.0 * M * N * K * cnt / (ms * 1e-3) / 1e12
        table.append({"M": M, "N": N, "K": K, "layout": "wgrad" if at else ("dgrad" if bt else "forward"),
                      "epilogue": EPI_NAMES.get(epi, str(epi)), "launches_per_step": cnt // steps,
                      "avg_us": round(ms * 1e3 / cnt, 1), "TFLOP/s": round(tf, 1),
                      "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 3)})
    out = {"bound": "mfma", "kernel": "gemm_bf16_w4_kernel (forward products) + gemm_bf16_k32_kernel (dgrad, wgrad)",
           "achieved": round(achieved, 1),
           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
           "traffic": measured_traffic(workload), "launches_per_step": launches // steps,
           "avg_launch_us": round(tot_ms * 1e3 / launches, 1), "flops_per_launch": tot_fl / launches,
           "gemm_share_of_step": round(tot_ms / steps / ms_per_step, 3),
           "ms_per_step_instrumented_build": round(ms_hooks, 4), "by_shape": table}
    att = attainable_peak()
    if att:
        out["attainable_peak"] = att
        out["frac_of_attainable"] = round(achieved / att, 4)
    if table:
        out["operand_data"] = gemm_on_constant_operands(table[0]["M"], table[0]["N"], table[0]["K"])
    return out


def gemm_on_constant_operands(M, N, K):
    """The step's most expensive product (forward layout, plain store) on random and on all-zero operands: the same
    instructions over the same addresses; what differs is the switching activity, hence the clock the chip holds
    under its power limit.  Context for `frac`, not part of it."""
    import torch
    import paper_2301_11913_amd as sw
    lib = sw.load_hooks_library()
    lib.swarm_kernel_gemm.restype = C.c_int
    lib.swarm_kernel_gemm.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_void_p]
    bf = torch.bfloat16
    out = {"M": M, "N": N, "K": K, "layout": "forward", "epilogue": "store"}
    Cm = torch.empty(M, N, device="cuda", dtype=bf)
    for name, fill in (("random", lambda *sh: torch.randn(*sh, device="cuda").to(bf)),
                       ("zeros", lambda *sh: torch.zeros(*sh, device="cuda", dtype=bf))):
        A, W = fill(M, K), fill(N, K)
        f = lambda: lib.swarm_kernel_gemm(1, M, N, K, A.data_ptr(), K, 0, W.data_ptr(), K, 0, Cm.data_ptr(), N, 0, None,
                                          None, 0, None, 0, None)
        for _ in range(3):
            if f() != 0:
                return None
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            f()
        e1.record()
        torch.cuda.synchronize()
        tf = 2.0 * M * N * K * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12
        out[name + "_TFLOP/s"] = round(tf, 1)
        out[name + "_frac"] = round(tf / MFMA_BF16_PEAK_TFLOPS, 3)
        del A, W
    return out


def codec_rates(wl, x_src, modes):
    """The stand-alone codec kernels on the workload's boundary tensor: HBM-cold (rotating through > 1.5 GiB of
    buffer sets, beyond the 256 MB last-level cache) and cache-warm (one buffer set).  Algorithmic bytes: element +
    code + scale / 64.  Times are launch-inclusive (back-to-back launches between two events on the launch stream);
    the kernel durations that rocprofv3 reports for the same launches are in profiles/ and are attached when there."""
    import torch
    import paper_2301_11913_amd as sw
    dev = x_src.device
    n = x_src.numel()
    es = x_src.element_size()
    byts = n * (es + 1 + 4.0 / 64)
    nset = max(2, int((1.5 * (1 << 30)) // byts) + 1) if "cold" in modes else 1
    xs = [torch.empty_like(x_src).copy_(x_src) for _ in range(nset)]
    cs = [torch.empty(n, dtype=torch.int8, device=dev) for _ in range(nset)]
    ss = [torch.empty(n // 64, dtype=torch.float32, device=dev) for _ in range(nset)]
    codec = {"elements": n, "bytes_per_call": byts, "peak_GBps": HBM_PEAK_GBS}
    for name, fn in (("encode", lambda i: sw.swarm_codec_encode(xs[i], cs[i], ss[i])),
                     ("decode", lambda i: sw.swarm_codec_decode(cs[i], ss[i], xs[i]))):
        for mode in modes:
            idx = list(range(nset)) * 3 if mode == "cold" else [0] * 50
            for i in idx[:nset]:
                fn(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in idx:
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / len(idx)
            codec["%s_%s_us" % (name, mode)] = round(us, 2)
            codec["%s_%s_GBps" % (name, mode)] = round(byts / us / 1e3, 1)
    if "cold" in modes:
        codec["frac_of_hbm_peak_cold"] = {"encode": round(codec["encode_cold_GBps"] / HBM_PEAK_GBS, 3),
                                          "decode": round(codec["decode_cold_GBps"] / HBM_PEAK_GBS, 3)}
    try:
        with open(os.path.join(ROOT, "profiles", "codec_%s_kernel_durations.json" % wl.name)) as f:
            codec["rocprofv3_kernel_durations"] = json.load(f)
    except (OSError, ValueError):
        pass
    return codec


def blas_threads():
    """Threads of the BLAS that numpy's matmul actually uses (the oracle's only library primitive)."""
    try:
        from threadpoolctl import threadpool_info
        n = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    return os.cpu_count() or 1


def model_flops(wl):
    """Paper convention (Table 6: 6 * parameters * tokens for fwd+bwd) plus the causal attention term."""
    T, d, f, S, B = wl.tokens, wl.d_model, wl.d_ffn, wl.seq, wl.batch
    gemm = 2.0 * T * (4 * d * d + (3 if wl.block == "rotary_geglu" else 2) * d * f)
    attn = 2.0 * B * wl.n_heads * wl.d_head * S * (S + 1)
    return 3.0 * (gemm + attn) * wl.n_layers * wl.n_repeat


def cpu_baseline(wl):
    """The oracle as it stands, on the host cores, on bounded samples of the workload.  `value`: one sequence
    (batch 1) through ONE block application, forward + recomputing backward (+ the codec on that sequence's
    boundary tensors), in fp32 with all BLAS threads, scaled to the workload's block count.  Beside it: the same
    sample in fp64, a 512-token sample on one thread, and the oracle codec's own rate."""
    import numpy as np
    import swarm_synth as synth
    from oracle import stage as osg, codec as ocodec
    from threadpoolctl import threadpool_limits
    apps = wl.n_layers * wl.n_repeat

    def run(seq, dt):
        sample = wl.replace(batch=1, seq=seq, n_layers=1, n_repeat=1)
        params, x, G = synth.make_params(sample), synth.make_x_in(sample), synth.make_grad_out(sample)
        t0 = time.perf_counter()
        if wl.boundary_codec:
            cx, sx = ocodec.encode(x.reshape(-1))
            x = ocodec.bf16_bits_to_f32(ocodec.decode(cx, sx, out="bf16")).reshape(x.shape)
            cg, sg = ocodec.encode(G.reshape(-1))
            G = ocodec.bf16_bits_to_f32(ocodec.decode(cg, sg, out="bf16")).reshape(G.shape)
        y = osg.stage_forward(params, x, sample.n_heads, 1, sample.ln_eps, dt, kind=sample.block)
        grads = osg.zero_grads(params, dt)
        gin = osg.stage_backward(params, x, G, grads, sample.n_heads, 1, sample.ln_eps, dt, kind=sample.block)
        if wl.boundary_codec:
            ocodec.encode(y.astype(np.float32).reshape(-1))
            ocodec.encode(gin.astype(np.float32).reshape(-1))
        return time.perf_counter() - t0

    seq = min(wl.seq, 2048)
    cores = blas_threads()
    if 96.0 * wl.tokens * wl.d_model * wl.d_model * apps < 2e12:
        # small workloads (the fp32 block, the d_model 1024 stage and block): the WHOLE workload, median of three runs
        def full(dt):
            params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
            ts = []
            for _ in range(3):
                t0 = time.perf_counter()
                osg.stage_forward(params, x, wl.n_heads, wl.n_repeat, wl.ln_eps, dt, kind=wl.block)
                osg.stage_backward(params, x, G, osg.zero_grads(params, dt), wl.n_heads, wl.n_repeat, wl.ln_eps, dt,
                                   kind=wl.block)
                ts.append(time.perf_counter() - t0)
            return sorted(ts)[1]
        t32, t64 = full(np.float32), full(np.float64)
        with threadpool_limits(limits=1):
            t1 = full(np.float32)
        return {"value": wl.tokens / t32, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                "sample": "fp32 numpy oracle, the whole workload (%d tokens, %d block applications, fwd + recomputing "
                          "bwd), median of 3 runs: %.2f s on %d BLAS threads" % (wl.tokens, apps, t32, cores),
                "fp64_all_cores_tokens_per_s": wl.tokens / t64, "fp32_one_thread_tokens_per_s": wl.tokens / t1}
    t32 = run(seq, np.float32)
    t64 = run(seq, np.float64)
    small = min(seq, 512)
    with threadpool_limits(limits=1):
        t1 = run(small, np.float32)
    # the oracle codec alone (numpy, one thread): bytes moved = element + code + scale / 64, as for the GPU figure
    xs = synth.make_x_in(wl.replace(batch=1, seq=seq)).reshape(-1)
    es = 2 if wl.dtype == "bf16" else 4
    t0 = time.perf_counter(); codes, scales = ocodec.encode(xs); te = time.perf_counter() - t0
    t0 = time.perf_counter(); ocodec.decode(codes, scales, out="bf16" if wl.dtype == "bf16" else "f32"); td = time.perf_counter() - t0
    byts = xs.size * (es + 1 + 4.0 / 64)
    return {"value": seq / (t32 * apps), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "fp32 numpy oracle, 1 sequence of %d tokens through 1 of %d block applications (fwd + "
                      "recomputing bwd%s), %.1f s on %d BLAS threads; rate divided by the block count"
                      % (seq, apps, " + codec" if wl.boundary_codec else "", t32, cores),
            "fp64_all_cores_tokens_per_s": seq / (t64 * apps), "fp64_sample_s": round(t64, 2),
            "fp32_one_thread_tokens_per_s": small / (t1 * apps),
            "one_thread_sample": "1 sequence of %d tokens, %.1f s" % (small, t1),
            "codec_encode_GBps": byts / te / 1e9, "codec_decode_GBps": byts / td / 1e9,
            "codec_sample": "oracle codec on %d elements, encode %.2f s, decode %.2f s" % (xs.size, te, td)}


def bench_boundary(args):
    """Workloads of the compression-aware boundary layers: one step = sender forward + backward and receiver
    forward + backward on one microbatch (both halves of a boundary, as the two neighbouring stages run them)."""
    import numpy as np
    import torch
    import swarm_synth as synth
    import paper_2301_11913_amd as sw
    wl = synth.BOUNDARY_WORKLOADS[args.workload]
    lib = sw.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)
    rn = lambda shape, std, mean=0.0: (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * std + mean).to(dt)
    T, m, c = wl.tokens, wl.d_model, wl.d_comp
    comp = {"ln_g": rn((m,), 0.02, 1.0), "ln_b": rn((m,), 0.02)}
    if wl.kind == "bottleneck":
        comp["w_c"] = rn((c, m), 0.02)
    dec = {"ln_g": rn((c,), 0.02, 1.0), "ln_b": rn((c,), 0.02), "w_d": rn((m, c), 0.02)}
    gc = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in comp.items()}
    gd = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in dec.items()}
    y, dx = rn((T, m), 1.0), rn((T, m), wl.grad_sigma)
    z, dz, x, dy = (torch.empty(s, dtype=dt, device=dev) for s in ((T, c), (T, c), (T, m), (T, m)))
    cfg = sw.BoundaryConfig(m, c, wl.kind, T, wl.dtype, wl.ln_eps)
    ws = torch.empty(max(sw.swarm_boundary_workspace_bytes(cfg, d, b) for d in (False, True) for b in (False, True)),
                     dtype=torch.uint8, device=dev)

    def step():
        sw.swarm_compress_forward(cfg, comp, y, z, ws)            # sending stage
        sw.swarm_decompress_forward(cfg, dec, z, x, ws)           # receiving stage
        sw.swarm_decompress_backward(cfg, dec, z, dx, dz, gd, ws)
        sw.swarm_compress_backward(cfg, comp, y, dz, dy, gc, ws)

    ms_per_step, ms_median, ms_min = timed_steps(step, args.steps, args.warmup)
    roofline = gemm_roofline(step, args.steps, ms_per_step, wl.name)
    out = {"metric": "boundary layer fwd+bwd tokens/s (sender + receiver halves)",
           "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
           "ms_per_step_min": round(ms_min, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
           "config": {"workload": wl.name, "kind": wl.kind, "d_model": m, "d_comp": c, "tokens": T},
           "roofline": roofline}
    if not args.no_cpu_baseline:
        from oracle import boundary as ob
        sample = wl.replace(tokens=min(T, 2048))
        cp, dp = synth.make_boundary_params(sample)
        ys, dzs, zs, dxs = synth.make_boundary_inputs(sample)
        t0 = time.perf_counter()
        zz = ob.compress_forward(ys, cp, wl.kind, c, wl.ln_eps)
        ob.decompress_forward(zz, dp, wl.ln_eps)
        dzz = ob.decompress_backward(zz, dxs, dp, {k: np.zeros(v.shape) for k, v in dp.items()}, wl.ln_eps)
        ob.compress_backward(ys, dzz, cp, {k: np.zeros(v.shape) for k, v in cp.items()}, wl.kind, c, wl.ln_eps)
        dts = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample.tokens / dts, "unit": "tokens/s", "cores": blas_threads(),
                               "kind": "oracle", "sample": "fp64 numpy oracle, %d tokens through both halves "
                               "(fwd + recomputing bwd), %.1f s" % (sample.tokens, dts)}
    print(json.dumps(out))


def bench_head(args):
    """Workload of the first / last stage extras: one step = embedding forward + backward (first stage) and
    head loss + backward (last stage) on one microbatch."""
    import numpy as np
    import torch
    import swarm_synth as synth
    import paper_2301_11913_amd as sw
    wl = synth.HEAD_WORKLOADS[args.workload]
    lib = sw.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)
    rn = lambda shape, std, mean=0.0: (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * std + mean).to(dt)
    T, d, V, Vp = wl.tokens, wl.d_model, wl.vocab, wl.vocab_rows
    table, w = rn((Vp, d), 0.02), rn((Vp, d), 0.02)
    table[V:] = 0; w[V:] = 0
    head = {"ln_g": rn((d,), 0.02, 1.0), "ln_b": rn((d,), 0.02), "w_vocab": w}
    grads = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in head.items()}
    grad_table = torch.zeros((Vp, d), dtype=torch.float32, device=dev)
    tok_np, tgt_np, _, _ = synth.make_head_inputs(wl.replace(d_model=8))      # ids only (log-uniform ranks)
    tokens, targets = torch.from_numpy(tok_np).to(dev), torch.from_numpy(tgt_np).to(dev)
    x_emb = torch.empty((T, d), dtype=dt, device=dev)
    x_head, dx_emb = rn((T, d), 1.0), rn((T, d), 1e-2)
    dx_head = torch.empty((T, d), dtype=dt, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    cfg = sw.HeadConfig(d, V, Vp, T, wl.dtype, wl.ln_eps)
    ws = torch.empty(sw.swarm_head_workspace_bytes(cfg, True), dtype=torch.uint8, device=dev)

    def step():
        sw.swarm_embedding_forward(tokens, table, V, x_emb)                               # first stage
        sw.swarm_head_loss_backward(cfg, head, x_head, targets, loss, None, dx_head, grads, ws)   # last stage
        sw.swarm_embedding_backward(tokens, dx_emb, V, grad_table)                        # first stage

    ms_per_step, ms_median, ms_min = timed_steps(step, args.steps, args.warmup)
    roofline = gemm_roofline(step, args.steps, ms_per_step, wl.name)
    out = {"metric": "embedding fwd+bwd and LM head loss+bwd tokens/s", "value": round(T / (ms_per_step * 1e-3), 1),
           "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
           "ms_per_step_min": round(ms_min, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": wl.dtype, "data": "synthetic",
           "config": {"workload": wl.name, "d_model": d, "vocab": V, "vocab_rows": Vp, "tokens": T},
           "loss": round(float(loss.item()), 4), "roofline": roofline}
    if not args.no_cpu_baseline:
        from oracle import head as oh
        sample = wl.replace(tokens=min(T, 256))
        tab, hp = synth.make_head_params(sample)
        tk, tg, xs, dxe = synth.make_head_inputs(sample)
        t0 = time.perf_counter()
        oh.embedding_forward(tk, tab)
        oh.head_loss_backward(xs, tg, hp, V, {k: np.zeros(v.shape) for k, v in hp.items()}, wl.ln_eps)
        oh.embedding_backward(tk, dxe, np.zeros(tab.shape))
        dts = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample.tokens / dts, "unit": "tokens/s", "cores": blas_threads(),
                               "kind": "oracle", "sample": "fp64 numpy oracle, %d tokens (embedding fwd + bwd, head "
                               "loss + bwd), %.1f s" % (sample.tokens, dts)}
    print(json.dumps(out))


def bench_lamb(args):
    """Optimiser workload: one step = one LAMB update of every parameter tensor of a stage."""
    import numpy as np
    import torch
    import swarm_synth as synth
    import paper_2301_11913_amd as sw
    wl = synth.LAMB_WORKLOADS[args.workload]
    sw.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)
    sizes = [int(np.prod(s)) for s in wl.shapes]
    tensors = []
    for shape, n in zip(wl.shapes, sizes):
        w = torch.randn(n, generator=g, device=dev) * 0.02 + (1.0 if len(shape) == 1 else 0.0)
        tensors.append(dict(w=w, p=w.to(dt), g=torch.randn(n, generator=g, device=dev) * 1e-3,
                            m=torch.zeros(n, device=dev), v=torch.zeros(n, device=dev)))
    ws = torch.empty(max(sw.swarm_lamb_workspace_bytes(n) for n in sizes), dtype=torch.uint8, device=dev)
    t_step = [0]

    def step():
        t_step[0] += 1
        for t in tensors:
            sw.swarm_lamb_step(t["w"], t["p"], t["g"], t["m"], t["v"], t_step[0], ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # the largest tensor's update, timed with events on the launch stream (the binding launches on torch's current one)
    big = max(range(len(sizes)), key=lambda i: sizes[i])
    t, ev = tensors[big], [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                           for _ in range(args.steps)]
    for e0, e1 in ev:
        t_step[0] += 1
        e0.record()
        sw.swarm_lamb_step(t["w"], t["p"], t["g"], t["m"], t["v"], t_step[0], ws)
        e1.record()
    torch.cuda.synchronize()
    ms_big = sum(e0.elapsed_time(e1) for e0, e1 in ev) / len(ev)
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # per element: first pass reads w, g, m, v and writes m, v, u (28 B); update reads w, u, writes w and the copy
    bytes_per_elem = 28 + 12 + (2 if wl.dtype == "bf16" else 4)
    achieved = bytes_per_elem * sizes[big] / (ms_big * 1e-3) / 1e9
    n_total = sum(sizes)
    out = {"metric": "LAMB parameters updated per second", "value": round(n_total / (ms_per_step * 1e-3), 1),
           "unit": "parameters/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": wl.name, "tensors": len(sizes), "parameters": n_total, "param_copy": wl.dtype},
           "roofline": {"bound": "hbm", "kernel": "lamb_moments_kernel + lamb_ratio_kernel + lamb_apply_kernel",
                        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(achieved / HBM_PEAK_GBS, 4),
                        # measured bytes of one update of the largest tensor: first pass + update kernel
                        "traffic": (lambda a, b: None if a is None or b is None else a + b)(
                            measured_traffic(wl.name, "lamb_moments"), measured_traffic(wl.name, "lamb_apply")),
                        "elements": sizes[big], "bytes_per_element": bytes_per_elem, "avg_update_us": round(ms_big * 1e3, 1)}}
    if not args.no_cpu_baseline:
        from oracle.lamb import lamb_step
        n = 1 << 24
        w, gr = synth.make_lamb_tensor(wl, big, n)
        m, v = np.zeros(n), np.zeros(n)
        t0 = time.perf_counter()
        for k in range(1, 4):
            w, m, v, _ = lamb_step(w, gr, m, v, k)
        dts = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 3 * n / dts, "unit": "parameters/s", "cores": 1, "kind": "oracle",
                               "sample": "fp64 numpy oracle, 3 steps on the first %d elements of the largest tensor, "
                                         "%.1f s" % (n, dts)}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="e2e_bf16_d4096")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unfused-codec", action="store_true",
                    help="call swarm_codec_decode/encode around the stage instead of the *_coded entry points")
    ap.add_argument("--codec-only", choices=["cold", "warm"], default=None,
                    help="run only the stand-alone codec kernels on the workload's boundary tensor, HBM-cold or "
                         "cache-warm (for a rocprofv3 --kernel-trace run whose kernel durations are the codec figure)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library is the per-peer, single-GPU path of a SWARM stage; peers of a stage share "
              "nothing but the gradient all-reduce, which is outside it. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import swarm_synth as synth
    import paper_2301_11913_amd as sw

    if args.workload in synth.BOUNDARY_WORKLOADS:
        return bench_boundary(args)
    if args.workload in synth.HEAD_WORKLOADS:
        return bench_head(args)
    if args.workload in synth.LAMB_WORKLOADS:
        return bench_lamb(args)
    wl = synth.WORKLOADS[args.workload]
    lib = sw.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed)

    def rn(shape, std, mean=0.0):
        return (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * std + mean).to(dt)

    params = []
    for _ in range(wl.n_layers):
        p = {k: rn(s, 0.02, 1.0 if k in ("ln1_g", "ln2_g") else 0.0) for k, s in wl.param_shapes().items()}
        params.append(p)
    grads = [{k: torch.zeros(s, dtype=torch.float32, device=dev) for k, s in wl.param_shapes().items()}
             for _ in range(wl.n_layers)]
    shape = (wl.batch, wl.seq, wl.d_model)
    n = wl.tokens * wl.d_model
    x_src, g_src = rn(shape, 1.0), rn(shape, wl.grad_sigma)
    if args.codec_only:
        codec = codec_rates(wl, x_src, (args.codec_only,))
        m = args.codec_only
        print(json.dumps({"metric": "int8 boundary codec GB/s (%s)" % ("HBM-cold" if m == "cold" else "cache-warm"),
                          "value": codec["encode_%s_GBps" % m], "unit": "GB/s", "n_gpus": 1, "higher_is_better": True,
                          "dtype": wl.dtype, "data": "synthetic", "config": {"workload": wl.name, "mode": m},
                          "codec": codec}))
        return
    cfg = sw.StageConfig(wl.d_model, wl.n_heads, wl.d_ffn, wl.n_layers, wl.n_repeat, wl.batch, wl.seq, wl.dtype,
                         wl.ln_eps, wl.block)
    ws = torch.empty(max(sw.swarm_stage_coded_workspace_bytes(cfg, True), sw.swarm_stage_coded_workspace_bytes(cfg, False)),
                     dtype=torch.uint8, device=dev)
    x, G, y, gin = (torch.empty(shape, dtype=dt, device=dev) for _ in range(4))
    codes = {k: torch.empty(n, dtype=torch.int8, device=dev) for k in ("x", "g", "y", "gin")}
    scales = {k: torch.empty(n // 64, dtype=torch.float32, device=dev) for k in ("x", "g", "y", "gin")}
    if wl.boundary_codec:
        sw.swarm_codec_encode(x_src, codes["x"], scales["x"])
        sw.swarm_codec_encode(g_src, codes["g"], scales["g"])
    else:
        x.copy_(x_src)
        G.copy_(g_src)

    def step():
        if wl.boundary_codec and not args.unfused_codec:
            # decode / encode fused into the stage's first and last kernels (bit-identical to the separate calls)
            sw.swarm_stage_forward_coded(cfg, params, codes["x"], scales["x"], x, codes["y"], scales["y"], ws)
            sw.swarm_stage_backward_coded(cfg, params, x, codes["g"], scales["g"], codes["gin"], scales["gin"], grads,
                                          ws)
            return
        if wl.boundary_codec:
            sw.swarm_codec_decode(codes["x"], scales["x"], x)
            sw.swarm_codec_decode(codes["g"], scales["g"], G)
        sw.swarm_stage_forward(cfg, params, x, y, ws)
        sw.swarm_stage_backward(cfg, params, x, G, gin, grads, ws)
        if wl.boundary_codec:
            sw.swarm_codec_encode(y, codes["y"], scales["y"])
            sw.swarm_codec_encode(gin, codes["gin"], scales["gin"])

    ms_per_step, ms_median, ms_min = timed_steps(step, args.steps, args.warmup)

    roofline = gemm_roofline(step, args.steps, ms_per_step, wl.name) if wl.dtype == "bf16" else None

    codec = codec_rates(wl, x_src, ("cold", "warm"))
    # a peer decodes x_in and grad_out and encodes x_out and grad_in per microbatch (for the workloads whose step
    # runs without the codec this is the compute-to-boundary ratio of Section 3.1 on the same boundary tensor)
    codec["stage_time_over_codec_time"] = round(ms_per_step * 1e3 / (2 * codec["encode_cold_us"] + 2 * codec["decode_cold_us"]), 1)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    tokens_per_s = wl.tokens / (ms_per_step * 1e-3)
    out = {"metric": "stage fwd+bwd tokens/s (+ int8 boundary codec)", "value": round(tokens_per_s, 1),
           "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
           "ms_per_step_min": round(ms_min, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": wl.dtype, "data": "synthetic",
           "config": {"workload": wl.name, "block": wl.block, "d_model": wl.d_model, "n_heads": wl.n_heads, "d_ffn": wl.d_ffn,
                      "seq": wl.seq, "microbatch": wl.batch, "blocks": wl.n_layers, "repeat": wl.n_repeat,
                      "codec": ("int8 absmax block 64 on stage input/output and their gradients, "
                                + ("separate kernels" if args.unfused_codec else "fused into the stage boundary"))
                      if wl.boundary_codec else "none"},
           "model_tflops_per_s": round(model_flops(wl) / (ms_per_step * 1e-3) / 1e12, 1),
           "roofline": roofline, "codec": codec}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
