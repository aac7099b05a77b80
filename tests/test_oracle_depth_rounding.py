"""How far bf16 STORAGE alone moves the output of a deep stack (CPU, oracle code only).

The benchmark description states the 2e-2 max-normalised bar for bf16 stages of at most four block applications;
the Section 4.3 stage is sixteen applications deep.  This test rebuilds the oracle's block from the oracle's own
pieces with one extra step - every tensor that a bf16 implementation has to keep in memory (a, q, k, v, the softmax
weights, o, h, c, u, g, y) is rounded to bf16 once, all other arithmetic stays exact fp64 - and measures the deviation
from the unrounded oracle chain per depth.  It is what licenses the depth-scaled end-to-end tolerance of the 16-deep
GPU parity test (2e-2 * R / 4): no implementation that stores bf16 can meet 2e-2 at depth 16, and the deviation
grows no faster than linearly beyond the four applications the bar was stated for.

Width 512 with the weight scale raised by sqrt(4096 / 512), so that every branch has the gain it has in the
d_model = 4096 model (sums over the input dimension of N(0, 0.02) weights).
"""
import math

import numpy as np

from oracle import stage as osg
from oracle.codec import bf16_bits_to_f32, f32_to_bf16_bits

D, H, F, S, R = 512, 8, 2048, 256, 16
KIND = "rotary_geglu"


def _bf16(t):
    return bf16_bits_to_f32(f32_to_bf16_bits(t.astype(np.float32))).astype(np.float64)


def _params(rng):
    s = 0.02 * math.sqrt(4096 / D)
    n = lambda shape, std, mean=0.0: _bf16(rng.standard_normal(shape) * std + mean)
    return {"ln1_g": n(D, 0.02, 1.0), "ln1_b": n(D, 0.02), "w_qkv": n((3 * D, D), s), "b_qkv": n(3 * D, 0.02),
            "w_o": n((D, D), s), "b_o": n(D, 0.02), "ln2_g": n(D, 0.02, 1.0), "ln2_b": n(D, 0.02),
            "w_1": n((2 * F, D), s), "b_1": n(2 * F, 0.02), "w_2": n((D, F), 0.02 * math.sqrt(16384 / F)),
            "b_2": n(D, 0.02)}


def _block(x, p, store):
    """oracle.stage.block_forward spelled out from the oracle's pieces, `store` applied to every kept tensor."""
    dh = D // H
    a = store(osg.layernorm_fwd(x, p["ln1_g"], p["ln1_b"], 1e-5)[0])
    qkv = a @ p["w_qkv"].T + p["b_qkv"]
    q, k, v = (osg._split_heads(qkv[:, i * D:(i + 1) * D], 1, S, H, dh) for i in range(3))
    rope = osg.rotary_angles(S, dh, x.dtype)
    q, k, v = store(osg.rotary(q, *rope)), store(osg.rotary(k, *rope)), store(v)
    _, prob = osg.attention_fwd(q, k, v)
    o = store(osg._merge_heads(np.matmul(store(prob), v), 1, S, H, dh))
    h = store(x + o @ p["w_o"].T + p["b_o"])
    c = store(osg.layernorm_fwd(h, p["ln2_g"], p["ln2_b"], 1e-5)[0])
    u = store(c @ p["w_1"].T + p["b_1"])
    g = store(osg.gelu(u[:, :F]) * u[:, F:])
    return store(h + g @ p["w_2"].T + p["b_2"])


def test_bf16_storage_error_grows_with_depth():
    rng = np.random.default_rng(0)
    p = _params(rng)
    x0 = _bf16(rng.standard_normal((S, D)))
    # the spelled-out block IS the oracle's block
    y_ref, _ = osg.block_forward(x0, p, H, 1e-5, 1, S, KIND)
    assert np.max(np.abs(_block(x0, p, lambda t: t) - y_ref)) <= 1e-12 * np.max(np.abs(y_ref))
    ref, emu, errs = x0, x0, []
    for depth in range(1, R + 1):
        ref = _block(ref, p, lambda t: t)
        emu = _block(emu, p, _bf16)
        errs.append(float(np.max(np.abs(emu - ref)) / np.max(np.abs(ref))))
    chain = osg.stage_forward([p], x0[None], H, R, kind=KIND)[0]
    assert np.max(np.abs(ref - chain)) <= 1e-9 * np.max(np.abs(chain))
    print("bf16 storage alone, max-normalised deviation by depth:", ["%.1e" % e for e in errs])
    assert all(e <= 2e-2 for e in errs[:4])                 # the stated bar is attainable where it is stated
    assert errs[R - 1] > 2e-2                               # and is not at depth 16, by storage rounding alone
    assert all(errs[n - 1] <= 2e-2 * n / 4 for n in range(4, R + 1))   # at most linear growth beyond depth 4
    assert errs[R - 1] > 2 * errs[0]                        # it does grow
