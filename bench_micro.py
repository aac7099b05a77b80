#!/usr/bin/env python3
"""Micro-benchmarks behind the roofline discussion of the bf16 MFMA GEMM (one MI355X).

    python bench_micro.py [--what mfma,lds,valu,stamps,data,vendor] [--json PATH]

  mfma   : a loop of nothing but MFMAs on register operands, in the GEMM kernel's shape (8 wavefronts per workgroup,
           two per SIMD, 128 accumulator registers per lane), for both bf16 MFMA shapes and for constant and random
           operand bits; reports TFLOP/s and the clock the chip ran at (shader-cycle counter over the 100 MHz wall clock)
  lds    : a loop of nothing but LDS fragment reads in the GEMM kernel's two read shapes and swizzles (bytes per clock
           and compute unit)
  valu   : the GEMM epilogue's GeLU on register values, one workgroup per compute unit, with one and with two
           wavefronts per SIMD: what a lone wavefront per SIMD (the four-wavefront GEMM kernel) can issue
  stamps : the 256 x 256 GEMM kernel of the instrumented build with wall-clock stamps at four points of every workgroup
           (first loads | loop | epilogue | gap to the next workgroup on the same compute unit), on the three layouts
           at the config-5 shapes
  data   : the GEMM and the attention kernels as the stage calls them (config-5 shapes), timed on random operands, on
           all-zero and on all-one operands: same instruction stream, same memory traffic, different switching
           activity in the matrix pipes and on the data paths, hence a different clock
  vendor : the GEMM kernel (plain store) beside the ROCm BLAS that torch.matmul calls, same operands, same run,
           alternating, on the products of the config-5 stage, random and all-zero operands; context for the roofline
           fraction (what the vendor's kernels reach on this machine and this data), never on the stage path

Everything else runs through libswarm_hooks.so (the instrumented build); prints a Markdown summary, optionally a JSON file.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

NOMINAL_GHZ = 2.4
N_CU = 256


def _clock_ghz(clocks, per_xcd=False):
    c = clocks.cpu().numpy().reshape(-1, 4)
    wall = (c[:, 1] - c[:, 0]).astype(np.float64)          # 100 MHz ticks
    cyc = (c[:, 3] - c[:, 2]).astype(np.float64)
    ok = wall > 0
    if per_xcd:     # consecutive workgroups go to the eight XCDs round-robin
        x = np.arange(len(wall)) % 8
        return [round(float(np.median(cyc[ok & (x == i)] / wall[ok & (x == i)]) * 0.1), 3) for i in range(8)]
    return float(np.median(cyc[ok] / wall[ok]) * 0.1), float(np.median(wall[ok]) * 0.01)


def run_mfma(lib, out):
    lib.swarm_microbench_mfma_rate.restype = C.c_int
    lib.swarm_microbench_mfma_rate.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    wgs = N_CU * 4
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(wgs * 4, dtype=torch.int64, device="cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    rows = []
    for shape, name, per_iter in ((0, "16x16x32", 32 * 16384.0), (1, "32x32x16", 8 * 32768.0)):
        iters = 4000 if shape == 0 else 8000
        for kind in ("constant", "random"):
            if kind == "constant":
                ops = torch.full((8 * 12 * 64 * 8,), 1.0, dtype=torch.bfloat16, device="cuda")
            else:
                ops = torch.randn(8 * 12 * 64 * 8, generator=g, device="cuda").to(torch.bfloat16)
            st = torch.cuda.current_stream().cuda_stream
            call = lambda: lib.swarm_microbench_mfma_rate(shape, ops.data_ptr(), sink.data_ptr(), clocks.data_ptr(), iters, wgs, st)
            assert call() == 0
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                assert call() == 0
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 3
            tflops = per_iter * iters * 8 * wgs / (ms * 1e-3) / 1e12
            ghz, wg_us = _clock_ghz(clocks)
            rows.append({"mfma": name, "operands": kind, "TFLOP/s": round(tflops, 1), "ms": round(ms, 3),
                         "shader_clock_GHz": round(ghz, 3), "frac_of_2500": round(tflops / 2500.0, 3),
                         "shader_clock_GHz_per_xcd": _clock_ghz(clocks, per_xcd=True)})
    out["mfma_rate"] = rows
    out["attainable_tflops_random_16x16x32"] = next(r["TFLOP/s"] for r in rows if r["mfma"] == "16x16x32" and r["operands"] == "random")
    print("## MFMA rate on register operands (8 wavefronts per workgroup, 1024 workgroups)\n")
    print("| MFMA | operand bits | TFLOP/s | of 2500 | shader clock (GHz) |\n|---|---|---|---|---|")
    for r in rows:
        print("| v_mfma_f32_%s_bf16 | %s | %.1f | %.3f | %.3f |" % (r["mfma"], r["operands"], r["TFLOP/s"], r["frac_of_2500"], r["shader_clock_GHz"]))
    print("\nShader clock per XCD (workgroups i mod 8), GHz:\n")
    for r in rows:
        print("* %s, %s operands: %s" % (r["mfma"], r["operands"], r["shader_clock_GHz_per_xcd"]))
    print()


def run_lds(lib, out):
    lib.swarm_microbench_lds_read.restype = C.c_int
    lib.swarm_microbench_lds_read.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    wgs = N_CU * 2
    sink = torch.empty(wgs * 512, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(wgs * 4, dtype=torch.int64, device="cuda")
    iters = 20000
    rows = []
    for tr, name in ((0, "ds_read_b128"), (1, "ds_read_b64_tr_b16 x 2")):
        st = torch.cuda.current_stream().cuda_stream
        call = lambda: lib.swarm_microbench_lds_read(tr, sink.data_ptr(), clocks.data_ptr(), iters, wgs, st)
        assert call() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); assert call() == 0; e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        byts = 12.0 * 1024 * iters * 8 * wgs
        ghz, wg_us = _clock_ghz(clocks)
        # per compute unit: one workgroup's bytes over its own duration (wall clock) and the measured clock
        per_cu = 12.0 * 1024 * iters * 8 / (wg_us * 1e-6) / (ghz * 1e9)
        rows.append({"read": name, "TB/s_chip": round(byts / (ms * 1e-3) / 1e12, 1), "B_per_clk_per_CU": round(per_cu, 1),
                     "shader_clock_GHz": round(ghz, 3)})
    out["lds_read"] = rows
    print("## LDS fragment reads alone (8 wavefronts per compute unit, the GEMM kernel's addresses and swizzles)\n")
    print("| read | bytes / clock / CU | TB/s over the chip | shader clock (GHz) |\n|---|---|---|---|")
    for r in rows:
        print("| %s | %.1f | %.1f | %.3f |" % (r["read"], r["B_per_clk_per_CU"], r["TB/s_chip"], r["shader_clock_GHz"]))
    print("\nA 32-deep sub-step of the 256 x 256 GEMM tile reads 96 KiB per compute unit for 512 MFMA-cycles per SIMD x 2 "
          "wavefronts = 1024 cycles at full rate: 96 B/clk.\n")


def run_valu(lib, out):
    lib.swarm_microbench_valu_rate.restype = C.c_int
    lib.swarm_microbench_valu_rate.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    inp = torch.randn(4096, device="cuda")
    wgs, iters = 1024, 2000
    sink = torch.empty(wgs * 512, device="cuda")
    clocks = torch.zeros(wgs * 4, dtype=torch.int64, device="cuda")
    rows = []
    for w in (1, 2, 1, 2):
        call = lambda: lib.swarm_microbench_valu_rate(w, inp.data_ptr(), sink.data_ptr(), clocks.data_ptr(), iters, wgs, None)
        for _ in range(2):
            assert call() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); assert call() == 0; e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        ghz, _ = _clock_ghz(clocks)
        rows.append({"wavefronts_per_simd": w, "ms": round(ms, 3), "G_gelu_per_s": round(wgs * w * 256 * 8 * iters / ms / 1e6, 1),
                     "shader_clock_GHz": round(ghz, 3)})
    out["valu"] = rows
    print("## Vector arithmetic (the epilogue's GeLU on 8 register values per lane), one workgroup per compute unit\n")
    print("| wavefronts per SIMD | ms | 10^9 GeLU / s over the chip | shader clock (GHz) |")
    print("|---|---|---|---|")
    for r in rows:
        print("| %d | %.3f | %.1f | %.3f |" % (r["wavefronts_per_simd"], r["ms"], r["G_gelu_per_s"], r["shader_clock_GHz"]))
    print()


def run_stamps(lib, out):
    lib.swarm_kernel_gemm_stamped.restype = C.c_int
    lib.swarm_kernel_gemm_stamped.argtypes = [C.c_int] * 3 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                            C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                            C.c_void_p, C.c_void_p]
    rows = []
    print("## Phases of a 256 x 256 tile (wall-clock stamps in every workgroup, microseconds, mean over the tiles)\n")
    print("| product (M x N x K, layout, epilogue; wavefronts per tile) | kernel | first loads | loop (p10 - p90) | epilogue | "
          "gap to next workgroup | loop alone TFLOP/s | launch TFLOP/s | loop time by XCD (min - max) | "
          "last tile ends after first idle CU |\n|---|---|---|---|---|---|---|---|---|---|")
    # forward products run on the four-wavefront kernel; the instrumented library can send them to the
    # eight-wavefront one (same tile, same epilogue arithmetic), measured here beside it
    for (M, N, K, a_t, b_t, epi, label, four) in (
            (8192, 12288, 4096, 0, 0, 1, "forward, bias; 4", 1), (8192, 12288, 4096, 0, 0, 1, "forward, bias; 8", 0),
            (8192, 16384, 4096, 0, 0, 3, "forward, bias + GeLU; 4", 1), (8192, 16384, 4096, 0, 0, 3, "forward, bias + GeLU; 8", 0),
            (8192, 4096, 16384, 0, 0, 2, "forward, bias + residual; 4", 1),
            (8192, 4096, 16384, 0, 0, 2, "forward, bias + residual; 8", 0),
            (8192, 16384, 4096, 0, 1, 4, "dgrad, x GeLU'; 8", 1), (8192, 4096, 16384, 0, 1, 0, "dgrad, store; 8", 1),
            (16384, 4096, 8192, 1, 1, 5, "wgrad, fp32 +=; 8", 1)):
        lib.swarm_kernel_gemm_four_waves(four)
        g = torch.Generator(device="cuda"); g.manual_seed(M + K)
        rn = lambda *s: torch.randn(*s, generator=g, device="cuda").to(torch.bfloat16)
        A = rn(K, M) if a_t else rn(M, K)
        B = rn(K, N) if b_t else rn(N, K)
        Cd = torch.zeros((M, N), dtype=torch.float32 if epi == 5 else torch.bfloat16, device="cuda")
        bias, aux = rn(N), rn(M, N)
        nt = (M // 256) * (N // 256)
        ws = torch.zeros(nt * 16, dtype=torch.int64, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        call = lambda: lib.swarm_kernel_gemm_stamped(M, N, K, A.data_ptr(), A.shape[1], a_t, B.data_ptr(), B.shape[1], b_t,
                                                     Cd.data_ptr(), N, epi, bias.data_ptr(), aux.data_ptr(), N, ws.data_ptr(), st)
        for _ in range(4):
            assert call() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); assert call() == 0; e1.record()
        torch.cuda.synchronize()
        kern_us = e0.elapsed_time(e1) * 1e3
        t = ws.cpu().numpy().reshape(nt, 16)
        s = t[:, :4].astype(np.float64) * 0.01
        s -= s[:, 0].min()
        hw, xcc = t[:, 4], t[:, 5] & 0xF
        key = xcc * 4096 + ((hw >> 8) & 0xF) + (((hw >> 13) & 0x7) << 4) + (((hw >> 12) & 1) << 7)
        pro, loop, ep = s[:, 1] - s[:, 0], s[:, 2] - s[:, 1], s[:, 3] - s[:, 2]
        gaps, last_end = [], []
        for k in set(key.tolist()):
            idx = np.where(key == k)[0]
            idx = idx[np.argsort(s[idx, 0])]
            gaps += [s[b, 0] - s[a, 3] for a, b in zip(idx[:-1], idx[1:])]
            last_end.append(s[idx[-1], 3])
        by_x = [float(loop[xcc == x].mean()) for x in sorted(set(xcc.tolist()))]
        ghz = t[:, 8].astype(np.float64) / (loop * 1e3)                 # shader cycles in the loop / its wall time
        ghz_x = [float(ghz[xcc == x].mean()) for x in sorted(set(xcc.tolist()))]
        flops_tile = 2.0 * 256 * 256 * K
        r = {"product": "%d x %d x %d, %s" % (M, N, K, label), "kernel_us": round(kern_us, 1),
             "first_loads_us": round(pro.mean(), 2), "loop_us": round(loop.mean(), 1),
             "loop_p10_p90": [round(v, 1) for v in np.percentile(loop, [10, 90])], "epilogue_us": round(ep.mean(), 1),
             "gap_us": round(float(np.mean(gaps)), 2) if gaps else None,
             "loop_TFLOPs": round(flops_tile * N_CU / (loop.mean() * 1e-6) / 1e12, 1),
             "launch_TFLOPs": round(2.0 * M * N * K / (kern_us * 1e-6) / 1e12, 1),
             "loop_by_xcd": [round(min(by_x), 1), round(max(by_x), 1)], "loop_us_per_xcd": [round(v, 1) for v in by_x],
             "loop_clock_GHz_per_xcd": [round(v, 3) for v in ghz_x], "loop_clock_GHz": round(float(ghz.mean()), 3),
             "end_spread_us": round(max(last_end) - min(last_end), 1), "compute_units_seen": len(set(key.tolist()))}
        rows.append(r)
        print("| %s | %.1f | %.2f | %.1f (%.1f - %.1f) | %.1f | %s | %.1f | %.1f | %.1f - %.1f | %.1f |" % (
            r["product"], r["kernel_us"], r["first_loads_us"], r["loop_us"], *r["loop_p10_p90"], r["epilogue_us"],
            "%.2f" % r["gap_us"] if r["gap_us"] is not None else "-", r["loop_TFLOPs"], r["launch_TFLOPs"], *r["loop_by_xcd"],
            r["end_spread_us"]))
        del A, B, Cd, aux
    lib.swarm_kernel_gemm_four_waves(1)
    out["tile_phases"] = rows
    print("\nPer XCD (0-7): loop time in microseconds and the shader clock during the loop (shader cycles / wall time):\n")
    for r in rows:
        print("* %s: loop %s us; clock %s GHz" % (r["product"], r["loop_us_per_xcd"], r["loop_clock_GHz_per_xcd"]))
    print()


def run_data(lib, out):
    lib.swarm_kernel_gemm.restype = C.c_int
    lib.swarm_kernel_gemm.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_void_p]
    lib.swarm_kernel_attention_fwd.restype = C.c_int
    lib.swarm_kernel_attention_fwd.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p]
    lib.swarm_kernel_attention_bwd.restype = C.c_int
    lib.swarm_kernel_attention_bwd.argtypes = [C.c_int] + [C.c_void_p] * 6 + [C.c_int] * 4 + [C.c_void_p]
    bf = torch.bfloat16
    fills = (("random", lambda *sh: torch.randn(*sh, device="cuda").to(bf)),
             ("zeros", lambda *sh: torch.zeros(*sh, device="cuda", dtype=bf)),
             ("ones", lambda *sh: torch.ones(*sh, device="cuda", dtype=bf)),
             ("random again", lambda *sh: torch.randn(*sh, device="cuda").to(bf)))

    def timed(f, iters):
        for _ in range(5):
            assert f() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    rows = []
    M, N, K = 8192, 16384, 4096
    Bt, S, H, dh = 4, 2048, 32, 128
    d = H * dh
    for name, fill in fills:
        A, W, Cm = fill(M, K), fill(N, K), torch.empty(M, N, device="cuda", dtype=bf)
        gemm = lambda: lib.swarm_kernel_gemm(1, M, N, K, A.data_ptr(), K, 0, W.data_ptr(), K, 0, Cm.data_ptr(), N, 0,
                                             None, None, 0, None, 0, None)
        us_g = timed(gemm, 20)
        del A, W, Cm
        qkv, do = fill(Bt, S, 3 * d), fill(Bt, S, d)
        o = torch.empty(Bt, S, d, dtype=bf, device="cuda")
        lse, delta = torch.empty(Bt, H, S, device="cuda"), torch.empty(Bt, H, S, device="cuda")
        dqkv = torch.empty_like(qkv)
        fwd = lambda: lib.swarm_kernel_attention_fwd(1, qkv.data_ptr(), o.data_ptr(), lse.data_ptr(), Bt, S, H, dh, None)
        bwd = lambda: lib.swarm_kernel_attention_bwd(1, qkv.data_ptr(), o.data_ptr(), do.data_ptr(), lse.data_ptr(),
                                                     delta.data_ptr(), dqkv.data_ptr(), Bt, S, H, dh, None)
        us_f = timed(fwd, 30)
        us_b = timed(bwd, 15)
        rows.append({"operands": name, "gemm_us": round(us_g, 1), "gemm_TFLOPs": round(2.0 * M * N * K / us_g * 1e-6, 1),
                     "attention_fwd_us": round(us_f, 1), "attention_bwd_us": round(us_b, 1)})
    out["data"] = rows
    print("## Kernel time against operand data (same kernels, same shapes, same traffic)\n")
    print("GEMM %d x %d x %d (forward layout, plain store); causal attention B = %d, S = %d, H = %d, d_head = %d.\n"
          % (M, N, K, Bt, S, H, dh))
    print("| operands | GEMM us | GEMM TFLOP/s | attention forward us | attention backward us |")
    print("|---|---|---|---|---|")
    for r in rows:
        print("| %s | %.1f | %.1f | %.1f | %.1f |" % (r["operands"], r["gemm_us"], r["gemm_TFLOPs"],
                                                   r["attention_fwd_us"], r["attention_bwd_us"]))
    print()


def run_vendor(lib, out):
    lib.swarm_kernel_gemm.restype = C.c_int
    lib.swarm_kernel_gemm.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                      C.c_void_p, C.c_int, C.c_void_p]
    bf = torch.bfloat16
    stream = torch.cuda.current_stream().cuda_stream

    def timed(f, iters=12):
        for _ in range(4):
            f()
        torch.cuda.synchronize()
        ts = []
        for _ in range(iters):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); f(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3)
        ts.sort()
        return ts[len(ts) // 2]

    # (name, M, N, K, A stored [K, M], B stored [K, N])
    products = (("forward (FFN1)", 8192, 16384, 4096, 0, 0), ("forward (QKV)", 8192, 12288, 4096, 0, 0),
                ("forward (FFN2)", 8192, 4096, 16384, 0, 0), ("dgrad (FFN1)", 8192, 4096, 16384, 0, 1),
                ("dgrad (FFN2)", 8192, 16384, 4096, 0, 1), ("wgrad (FFN1)", 16384, 4096, 8192, 1, 1),
                ("wgrad (out-proj)", 4096, 4096, 8192, 1, 1))
    rows = []
    for name, M, N, K, a_t, b_t in products:
        for kind in ("random", "zeros"):
            mk = (lambda *sh: torch.randn(*sh, device="cuda").to(bf)) if kind == "random" else \
                 (lambda *sh: torch.zeros(*sh, device="cuda", dtype=bf))
            A = mk(K, M) if a_t else mk(M, K)
            B = mk(K, N) if b_t else mk(N, K)
            Co, Cv = torch.empty(M, N, device="cuda", dtype=bf), torch.empty(M, N, device="cuda", dtype=bf)
            Av = A.t() if a_t else A
            Bv = B if b_t else B.t()

            def ours():
                assert lib.swarm_kernel_gemm(1, M, N, K, A.data_ptr(), A.shape[1], a_t, B.data_ptr(), B.shape[1], b_t,
                                             Co.data_ptr(), N, 0, None, None, 0, None, 0, stream) == 0

            def vendor():
                torch.matmul(Av, Bv, out=Cv)

            us = [timed(ours), timed(vendor), timed(ours), timed(vendor)]
            if kind == "random":     # same product on both sides (fp32 accumulation, one bf16 rounding)
                diff = float((Co.float() - Cv.float()).abs().max() / Cv.float().abs().max())
            else:
                diff = 0.0
            fl = 2.0 * M * N * K * 1e-6
            rows.append({"product": name, "M": M, "N": N, "K": K, "operands": kind,
                         "this_us": [round(us[0], 1), round(us[2], 1)], "vendor_us": [round(us[1], 1), round(us[3], 1)],
                         "this_TFLOPs": round(fl / min(us[0], us[2]), 1), "vendor_TFLOPs": round(fl / min(us[1], us[3]), 1),
                         "max_normalised_difference": diff})
            del A, B, Co, Cv
    out["vendor"] = rows
    print("## This GEMM kernel beside the ROCm BLAS behind torch.matmul (same operands, same run, alternating)\n")
    print("bf16 in, fp32 accumulation, bf16 out, plain store; median of 12 launches, two rounds each, the better round "
          "counted; torch %s.\n" % torch.__version__)
    print("| product | M x N x K | operands | this kernel us | vendor us | this TFLOP/s (of 2500) | vendor TFLOP/s (of 2500) |")
    print("|---|---|---|---|---|---|---|")
    for r in rows:
        print("| %s | %d x %d x %d | %s | %s | %s | %.1f (%.3f) | %.1f (%.3f) |" % (
            r["product"], r["M"], r["N"], r["K"], r["operands"], " / ".join("%.1f" % v for v in r["this_us"]),
            " / ".join("%.1f" % v for v in r["vendor_us"]), r["this_TFLOPs"], r["this_TFLOPs"] / 2500.0,
            r["vendor_TFLOPs"], r["vendor_TFLOPs"] / 2500.0))
    print()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--what", default="mfma,lds,valu,stamps,data,vendor")
    ap.add_argument("--json", default=None)
    args = ap.parse_args()
    import paper_2301_11913_amd as sw
    lib = sw.load_hooks_library()
    torch.cuda.set_device(0)
    out = {}
    print("# Micro-benchmarks behind the GEMM roofline (MI355X; nominal %.1f GHz, 256 compute units)\n" % NOMINAL_GHZ)
    for w in args.what.split(","):
        {"mfma": run_mfma, "lds": run_lds, "valu": run_valu, "stamps": run_stamps, "data": run_data,
         "vendor": run_vendor}[w](lib, out)
    if args.json:
        with open(args.json, "w") as f:
            json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
