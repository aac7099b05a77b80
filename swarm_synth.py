"""Seeded synthetic inputs for the SWARM pipeline-stage workloads.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It holds none of the method's arithmetic: it only
names the workload shapes and draws tensors from a seeded generator.

Shapes follow the paper's layer descriptions (Section 4.2 and the appendix
"Additional Details for Section 4.1": the "xxlarge" layer is d_model 4096,
d_FFN 16384, 32 heads, sequence 512, microbatch 4; the large-scale run trains
on sequences of up to 2048 tokens).  The paper's own throughput runs feed
random samples, so no dataset is needed.

Distributions (per workload): x_in ~ N(0,1); weight matrices and all biases
~ N(0, 0.02); LayerNorm gains 1 + N(0, 0.02); grad_out ~ N(0, sigma_g).
Every tensor has its own seed derived from (workload seed, tensor name), so
generation order does not matter.  For bf16 workloads every tensor is rounded
to bf16 (round-to-nearest-even) on the host; the returned fp32 arrays then
hold exactly representable bf16 values, so both sides start from the same bits.
"""
from __future__ import annotations

import dataclasses
import math
import zlib

import numpy as np
import torch

BASE_SEED = 20230127

PARAM_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"
    d_model: int
    n_heads: int
    d_ffn: int
    seq: int
    batch: int
    n_layers: int         # L distinct parameter sets
    n_repeat: int         # R applications of each set in a row
    grad_sigma: float
    codec_block: int = 64
    ln_eps: float = 1e-5
    seed: int = BASE_SEED
    boundary_codec: bool = False   # stage entry/exit tensors travel as int8
    block: str = "gelu"            # "gelu" | "rotary_geglu" (w_1, b_1 then have 2*d_ffn rows: gate | up)

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    def param_shapes(self) -> dict:
        d, f = self.d_model, self.d_ffn
        f1 = 2 * f if self.block == "rotary_geglu" else f
        return {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (3 * d, d), "b_qkv": (3 * d,),
                "w_o": (d, d), "b_o": (d,), "ln2_g": (d,), "ln2_b": (d,),
                "w_1": (f1, d), "b_1": (f1,), "w_2": (d, f), "b_2": (d,)}

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def _wl(i, name, **kw):
    return Workload(name=name, seed=BASE_SEED + i, **kw)


# The five configurations the benchmark description names.
WORKLOADS = {
    "block_f32_d256": _wl(1, "block_f32_d256", dtype="f32", d_model=256, n_heads=4, d_ffn=1024,
                          seq=128, batch=4, n_layers=1, n_repeat=1, grad_sigma=1.0),
    "stage2_bf16_d1024": _wl(2, "stage2_bf16_d1024", dtype="bf16", d_model=1024, n_heads=16, d_ffn=4096,
                             seq=512, batch=8, n_layers=2, n_repeat=1, grad_sigma=1e-2),
    "width_bf16_d1024": _wl(3, "width_bf16_d1024", dtype="bf16", d_model=1024, n_heads=8, d_ffn=4096,
                            seq=512, batch=8, n_layers=1, n_repeat=1, grad_sigma=1e-2),
    "width_bf16_d2048": _wl(3, "width_bf16_d2048", dtype="bf16", d_model=2048, n_heads=16, d_ffn=8192,
                            seq=512, batch=8, n_layers=1, n_repeat=1, grad_sigma=1e-2),
    "width_bf16_d4096": _wl(3, "width_bf16_d4096", dtype="bf16", d_model=4096, n_heads=32, d_ffn=16384,
                            seq=512, batch=8, n_layers=1, n_repeat=1, grad_sigma=1e-2),
    "shared4_bf16_d4096": _wl(4, "shared4_bf16_d4096", dtype="bf16", d_model=4096, n_heads=32, d_ffn=16384,
                              seq=512, batch=4, n_layers=1, n_repeat=4, grad_sigma=1e-2),
    "e2e_bf16_d4096": _wl(5, "e2e_bf16_d4096", dtype="bf16", d_model=4096, n_heads=32, d_ffn=16384,
                          seq=2048, batch=4, n_layers=2, n_repeat=1, grad_sigma=1e-2,
                          boundary_codec=True),
    # the Section 4.3 model's stage: one shared rotary + GeGLU block (d_model 4096) applied 16 times,
    # sequences of up to 2048 tokens, one sequence per microbatch
    "shared16_rope_geglu_d4096": _wl(6, "shared16_rope_geglu_d4096", dtype="bf16", d_model=4096, n_heads=32,
                                     d_ffn=16384, seq=2048, batch=1, n_layers=1, n_repeat=16, grad_sigma=1e-2,
                                     block="rotary_geglu", boundary_codec=True),
}


def _tensor_seed(seed: int, name: str) -> int:
    return (seed * 1000003 + zlib.crc32(name.encode())) % (2 ** 63 - 1)


def normal(seed: int, name: str, shape, mean: float = 0.0, std: float = 1.0,
           bf16: bool = False) -> np.ndarray:
    """fp32 array of N(mean, std) draws; with bf16=True the values are rounded to bf16."""
    g = torch.Generator(device="cpu")
    g.manual_seed(_tensor_seed(seed, name))
    t = torch.randn(tuple(shape), generator=g, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    if bf16:
        t = t.to(torch.bfloat16).to(torch.float32)
    return t.numpy()


def make_params(wl: Workload) -> list:
    """List of L dicts (one per distinct block) of fp32 arrays."""
    bf = wl.dtype == "bf16"
    out = []
    for l in range(wl.n_layers):
        p = {}
        for k, shp in wl.param_shapes().items():
            if k in ("ln1_g", "ln2_g"):
                p[k] = normal(wl.seed, f"L{l}.{k}", shp, 1.0, 0.02, bf)
            else:
                p[k] = normal(wl.seed, f"L{l}.{k}", shp, 0.0, 0.02, bf)
        out.append(p)
    return out


def make_x_in(wl: Workload) -> np.ndarray:
    return normal(wl.seed, "x_in", (wl.batch, wl.seq, wl.d_model), 0.0, 1.0, wl.dtype == "bf16")


def make_grad_out(wl: Workload) -> np.ndarray:
    return normal(wl.seed, "grad_out", (wl.batch, wl.seq, wl.d_model), 0.0, wl.grad_sigma,
                  wl.dtype == "bf16")


def codec_tensor(seed: int, n_elems: int, std: float = 1.0, bf16: bool = False,
                 name: str = "codec") -> np.ndarray:
    """Flat tensor with the value distribution of a boundary activation."""
    return normal(seed, name, (n_elems,), 0.0, std, bf16)


# ----------------------------------------------------------------------------------------------------
# Compression-aware stage boundary (appendix "Compression-Aware Architectures"): the sending stage maps its
# output y [T, m] to z [T, c] (linear bottleneck or maxout), the receiving stage maps z back to [T, m].
@dataclasses.dataclass(frozen=True)
class BoundaryWorkload:
    name: str
    dtype: str            # "f32" | "bf16"
    kind: str             # "bottleneck" | "maxout"
    d_model: int          # m
    d_comp: int           # c (bottleneck) or m / k (maxout)
    tokens: int           # T = microbatch * sequence
    grad_sigma: float
    ln_eps: float = 1e-5
    seed: int = BASE_SEED + 100

    def replace(self, **kw) -> "BoundaryWorkload":
        return dataclasses.replace(self, **kw)


BOUNDARY_WORKLOADS = {
    # the appendix evaluates both layers at a compression factor of 2 on sequences of 2048 tokens
    "bottleneck2_bf16_d4096": BoundaryWorkload("bottleneck2_bf16_d4096", "bf16", "bottleneck", 4096, 2048, 8192, 1e-2,
                                               seed=BASE_SEED + 101),
    "maxout2_bf16_d4096": BoundaryWorkload("maxout2_bf16_d4096", "bf16", "maxout", 4096, 2048, 8192, 1e-2,
                                           seed=BASE_SEED + 102),
}


def make_boundary_params(wl: BoundaryWorkload):
    """(compress params, decompress params): fp32 arrays, bf16-rounded for bf16 workloads."""
    bf = wl.dtype == "bf16"
    m, c = wl.d_model, wl.d_comp
    comp = {"ln_g": normal(wl.seed, "c.ln_g", (m,), 1.0, 0.02, bf), "ln_b": normal(wl.seed, "c.ln_b", (m,), 0.0, 0.02, bf)}
    if wl.kind == "bottleneck":
        comp["w_c"] = normal(wl.seed, "c.w_c", (c, m), 0.0, 0.02, bf)
    dec = {"ln_g": normal(wl.seed, "d.ln_g", (c,), 1.0, 0.02, bf), "ln_b": normal(wl.seed, "d.ln_b", (c,), 0.0, 0.02, bf),
           "w_d": normal(wl.seed, "d.w_d", (m, c), 0.0, 0.02, bf)}
    return comp, dec


def make_boundary_inputs(wl: BoundaryWorkload):
    """y [T, m] (sender input), dz [T, c] (gradient arriving at the sender), z [T, c] (receiver input),
    dx [T, m] (gradient arriving at the receiver)."""
    bf = wl.dtype == "bf16"
    T, m, c = wl.tokens, wl.d_model, wl.d_comp
    return (normal(wl.seed, "y", (T, m), 0.0, 1.0, bf), normal(wl.seed, "dz", (T, c), 0.0, wl.grad_sigma, bf),
            normal(wl.seed, "z", (T, c), 0.0, 1.0, bf), normal(wl.seed, "dx", (T, m), 0.0, wl.grad_sigma, bf))


# ----------------------------------------------------------------------------------------------------
# First / last stage extras (Section 4.3): token embedding and language-modelling head + loss.
@dataclasses.dataclass(frozen=True)
class HeadWorkload:
    name: str
    dtype: str
    d_model: int
    vocab: int            # V: number of real tokens
    vocab_rows: int       # rows of the weight matrices (V padded to a tile multiple; rows >= V are padding)
    tokens: int           # T = microbatch * sequence
    ln_eps: float = 1e-5
    seed: int = BASE_SEED + 200

    def replace(self, **kw) -> "HeadWorkload":
        return dataclasses.replace(self, **kw)


HEAD_WORKLOADS = {
    # the Section 4.3 model: d_model 4096, the GPT-2 tokenizer's 50257 tokens, one 2048-token sequence per microbatch
    "head_gpt2vocab_bf16_d4096": HeadWorkload("head_gpt2vocab_bf16_d4096", "bf16", 4096, 50257, 50432, 2048,
                                              seed=BASE_SEED + 201),
}


def make_head_params(wl: HeadWorkload):
    """(embedding table [rows, d], head params ln_g, ln_b [d], w_vocab [rows, d]); padding rows are zero."""
    bf = wl.dtype == "bf16"
    d = wl.d_model
    table = normal(wl.seed, "table", (wl.vocab_rows, d), 0.0, 0.02, bf)
    w = normal(wl.seed, "w_vocab", (wl.vocab_rows, d), 0.0, 0.02, bf)
    table[wl.vocab:] = 0.0
    w[wl.vocab:] = 0.0
    head = {"ln_g": normal(wl.seed, "h.ln_g", (d,), 1.0, 0.02, bf), "ln_b": normal(wl.seed, "h.ln_b", (d,), 0.0, 0.02, bf),
            "w_vocab": w}
    return table, head


def make_head_inputs(wl: HeadWorkload):
    """tokens [T] and targets [T] (int32, Zipf-like: frequent ids repeat inside a microbatch, as in text),
    x [T, d] (input of the head), dx_emb [T, d] (gradient arriving at the embedding)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(_tensor_seed(wl.seed, "tokens"))
    u = torch.rand((2, wl.tokens), generator=g, dtype=torch.float64)
    ids = torch.floor(torch.exp(u * math.log(wl.vocab))).to(torch.int64).clamp_(1, wl.vocab) - 1   # log-uniform ranks
    bf = wl.dtype == "bf16"
    return (ids[0].to(torch.int32).numpy(), ids[1].to(torch.int32).numpy(),
            normal(wl.seed, "x", (wl.tokens, wl.d_model), 0.0, 1.0, bf),
            normal(wl.seed, "dx_emb", (wl.tokens, wl.d_model), 0.0, 1e-2, bf))


# Optimiser step (appendix "Additional Details for Section 4.3"): LAMB over the parameter tensors of one stage.
@dataclasses.dataclass(frozen=True)
class LambWorkload:
    name: str
    dtype: str            # type of the stage's copy of the weights (master weights and moments are fp32)
    shapes: tuple         # one entry per parameter tensor
    seed: int = BASE_SEED + 300


def _rope_geglu_block_shapes(d: int, f: int):
    return ((d,), (d,), (3 * d, d), (3 * d,), (d, d), (d,), (d,), (d,), (2 * f, d), (2 * f,), (d, f), (d,))


LAMB_WORKLOADS = {
    # the tensors of the Section 4.3 stage (one shared rotary + GeGLU block, d_model 4096, d_ffn 16384)
    "lamb_stage_rope_geglu_d4096": LambWorkload("lamb_stage_rope_geglu_d4096", "bf16",
                                                _rope_geglu_block_shapes(4096, 16384), seed=BASE_SEED + 301),
}


def make_lamb_tensor(wl: LambWorkload, index: int, n: int = None):
    """(w, grad) fp32 of tensor `index` (flattened, optionally only the first n elements' worth): weights
    N(0, 0.02) (vectors: about 1), gradients N(0, 1e-3) as after averaging over a large batch."""
    shape = wl.shapes[index]
    n = int(np.prod(shape)) if n is None else n
    w = normal(wl.seed, "lamb.w%d" % index, (n,), 1.0 if len(shape) == 1 else 0.0, 0.02, False)
    g = normal(wl.seed, "lamb.g%d" % index, (n,), 0.0, 1e-3, False)
    return w, g
