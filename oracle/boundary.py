"""CPU oracle for the compression-aware stage-boundary layers.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (paper_2301_11913_amd/, bench.py's timed region)
imports this module; it exists to check the HIP kernels.

What it computes (appendix "Compression-Aware Architectures", paragraphs "Bottleneck layers" and "Maxout
compression"): the two halves of a compressed stage boundary.  With y [T, m] the output of the sending stage's
last layer:

    sender   (holds w_c):   z = LayerNorm(y) w_c                      bottleneck, z [T, c], c < m
                            z = maxout_k(LayerNorm(y))                maxout, z [T, m/k]
    receiver (holds w_d):   x = LayerNorm(z) w_d                      x [T, m]

so that receiver(sender(y)) is the paper's LayerNorm(LayerNorm(MLP) w_c) w_d, resp.
LayerNorm(maxout_k(LayerNorm(MLP))) w_d; z is what crosses the network (m/c resp. k times fewer values, and it
may additionally go through the int8 codec).  maxout_k takes the maximum over each non-overlapping window of k
consecutive features.

Readings where the paper is silent: the LayerNorms have learned gain and bias and the same eps-inside-the-root
form as the block's; the two linear maps have no bias (the appendix writes its formulas without biases);
weights are stored [out, in] like every other matrix of the library (w_c [c, m], w_d [m, c]); in the maxout
backward a tie goes to the first maximal feature of the window.

Plain numpy; np.matmul is the only library primitive.  Pins (tests/test_oracle_boundary.py): central finite
differences, a PyTorch autograd re-statement (nn.functional.layer_norm, max over a reshaped axis), maxout special
cases (k = 1, sorted windows, gradient mass), and the data-transfer factor of the appendix's table.
"""
from __future__ import annotations

import numpy as np

from oracle.stage import layernorm_fwd, layernorm_bwd


def maxout_fwd(a, k):
    """a [T, m] -> (z [T, m/k], index of the first maximum in each window)."""
    T, m = a.shape
    w = a.reshape(T, m // k, k)
    idx = w.argmax(axis=-1)                      # numpy returns the first maximum
    return np.take_along_axis(w, idx[..., None], axis=-1)[..., 0], idx


def maxout_bwd(dz, idx, k):
    """dz [T, m/k] -> da [T, m]: the gradient goes to the window's (first) maximal feature."""
    T, n = dz.shape
    da = np.zeros((T, n, k), dtype=dz.dtype)
    np.put_along_axis(da, idx[..., None], dz[..., None], axis=-1)
    return da.reshape(T, n * k)


# ------------------------------------------------------------------------------------------- sender
def _stored(a, store):
    """a as the kernel holds it in memory: None = exact, "f32" / "bf16" = rounded to that type (nearest even)."""
    if store is None:
        return a
    a32 = a.astype(np.float32)
    if store == "bf16":
        from oracle.codec import f32_to_bf16_bits, bf16_bits_to_f32
        a32 = bf16_bits_to_f32(f32_to_bf16_bits(a32))
    return a32.astype(a.dtype)


def compress_forward(y, p, kind, d_comp, eps=1e-5, dt=np.float64, keep=False, store=None):
    """y [T, m] -> z [T, d_comp].  p: ln_g, ln_b [m] and, for the bottleneck, w_c [d_comp, m].

    `store`: maxout picks one feature per window, a discrete decision taken on floating-point values; a parity
    test passes the storage type of the kernel under test so that both sides decide on the same numbers (the
    normalised row rounded to that type).  It only matters for near-ties."""
    y = np.asarray(y, dtype=dt)
    a, xhat, r = layernorm_fwd(y, np.asarray(p["ln_g"], dt), np.asarray(p["ln_b"], dt), eps)
    if kind == "bottleneck":
        z, idx = a @ np.asarray(p["w_c"], dt).T, None
    elif kind == "maxout":
        z, idx = maxout_fwd(_stored(a, store), y.shape[1] // d_comp)
    else:
        raise ValueError(kind)
    return (z, dict(a=a, xhat=xhat, r=r, idx=idx)) if keep else z


def compress_backward(y, dz, p, grads, kind, d_comp, eps=1e-5, dt=np.float64, store=None):
    """Recomputes the forward from y; returns dy [T, m] and ADDS the parameter gradients into `grads`."""
    _, c = compress_forward(y, p, kind, d_comp, eps, dt, keep=True, store=store)
    dz = np.asarray(dz, dtype=dt)
    if kind == "bottleneck":
        grads["w_c"] += dz.T @ c["a"]
        da = dz @ np.asarray(p["w_c"], dt)
    else:
        da = maxout_bwd(dz, c["idx"], np.shape(y)[1] // d_comp)
    dy, dg, db = layernorm_bwd(da, c["xhat"], c["r"], np.asarray(p["ln_g"], dt))
    grads["ln_g"] += dg
    grads["ln_b"] += db
    return dy


# ------------------------------------------------------------------------------------------- receiver
def decompress_forward(z, p, eps=1e-5, dt=np.float64, keep=False):
    """z [T, c] -> x [T, m].  p: ln_g, ln_b [c], w_d [m, c]."""
    z = np.asarray(z, dtype=dt)
    n, xhat, r = layernorm_fwd(z, np.asarray(p["ln_g"], dt), np.asarray(p["ln_b"], dt), eps)
    x = n @ np.asarray(p["w_d"], dt).T
    return (x, dict(n=n, xhat=xhat, r=r)) if keep else x


def decompress_backward(z, dx, p, grads, eps=1e-5, dt=np.float64):
    """Recomputes the forward from z; returns dz [T, c] and ADDS the parameter gradients into `grads`."""
    _, c = decompress_forward(z, p, eps, dt, keep=True)
    dx = np.asarray(dx, dtype=dt)
    grads["w_d"] += dx.T @ c["n"]
    dn = dx @ np.asarray(p["w_d"], dt)
    dz, dg, db = layernorm_bwd(dn, c["xhat"], c["r"], np.asarray(p["ln_g"], dt))
    grads["ln_g"] += dg
    grads["ln_b"] += db
    return dz
