"""Build the two gfx950 libraries in-tree with hipcc.

    python -m paper_2301_11913_amd.build

libswarm_stage.so is the product: every translation unit under csrc/ except the hook files, compiled to an object
under _build/ and linked.  libswarm_hooks.so is the instrumented build for tests and measurements: the same objects,
with the GEMM sources compiled a second time under -DSWARM_KERNEL_HOOKS (per-launch event timer, optional phase
stamps), plus kernel_hooks.hip (single-kernel entry points) and microbench.hip.  hipcc cross-compiles, so no GPU is
needed to build.
"""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libswarm_stage.so")
OUT_HOOKS = os.path.join(PKG, "libswarm_hooks.so")
BUILD_DIR = os.path.join(ROOT, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
          "-I", CSRC, "-Wall", "-Wno-unused-function",
          # packed-fp32 instructions are kept out of all device code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# per-file extras: the codec must not contract a*b+c or relax division
EXTRA = {"codec.hip": ["-ffp-contract=off"]}


# files that exist only in the instrumented build, and files that are compiled a second time for it
HOOK_ONLY = ("kernel_hooks.hip", "microbench.hip")
HOOK_VARIANTS = ("gemm_bf16.hip", "gemm_bf16_dma.hip")


def _compile(job) -> str:
    src, hooks = job
    obj = _obj(src, hooks)
    cmd = [HIPCC, "-c", src, "-o", obj] + COMMON + EXTRA.get(os.path.basename(src), [])
    if hooks:
        cmd.append("-DSWARM_KERNEL_HOOKS")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, " ".join(cmd), r.stderr[-8000:]))
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    return warn


def _obj(src: str, hooks: bool) -> str:
    return os.path.join(BUILD_DIR, os.path.basename(src) + (".hooks.o" if hooks else ".o"))


def _link(out: str, objs) -> None:
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out] + list(objs)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr[-8000:])


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    name = os.path.basename
    # longest translation units first, so the pool does not end on one of them
    jobs = [(s, True) for s in srcs if name(s) in HOOK_VARIANTS] + \
           [(s, False) for s in srcs if name(s) not in HOOK_ONLY] + [(s, True) for s in srcs if name(s) in HOOK_ONLY]
    jobs.sort(key=lambda j: -os.path.getsize(j[0]))
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        for (src, hooks), warn in zip(jobs, ex.map(_compile, jobs)):
            if verbose and warn:
                print("[%s%s]\n%s" % (name(src), " (hooks)" if hooks else "", warn), file=sys.stderr)
    product = [s for s in srcs if name(s) not in HOOK_ONLY]
    _link(OUT, [_obj(s, False) for s in product])
    _link(OUT_HOOKS, [_obj(s, name(s) in HOOK_VARIANTS) for s in product] + [_obj(s, True) for s in srcs if name(s) in HOOK_ONLY])
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
