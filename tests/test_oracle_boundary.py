"""Pins for the boundary-layer oracle (oracle/boundary.py).  CPU only.

Independent references: central finite differences (fp64); a PyTorch autograd re-statement built from
torch.nn.functional.layer_norm, a bias-free linear map and a max over a reshaped axis; maxout special cases with
known answers; the data-transfer factor printed in the compression appendix's table.
"""
import os

import numpy as np
import pytest
import torch

from oracle import boundary as ob
import swarm_synth as synth

HERE = os.path.dirname(__file__)


def _tiny(kind, m=24, c=8, T=7, seed=5):
    wl = synth.BoundaryWorkload("tiny", "f32", kind, m, c, T, 1.0, seed=seed)
    comp, dec = synth.make_boundary_params(wl)
    for p in (comp, dec):            # more signal than the workloads' 0.02 so every path shows in the FD check
        for k in p:
            if k.startswith("w_") or k == "ln_b":
                p[k] = p[k] * 15.0
    return wl, comp, dec, synth.make_boundary_inputs(wl)


def _fd(f, arr, eps=1e-6):
    g = np.zeros_like(arr, dtype=np.float64)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = arr[i]
        arr[i] = old + eps; fp = f()
        arr[i] = old - eps; fm = f()
        arr[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


@pytest.mark.parametrize("kind", ["bottleneck", "maxout"])
def test_compress_backward_matches_finite_differences(kind):
    wl, comp, _, (y, dz, _, _) = _tiny(kind)
    comp = {k: v.astype(np.float64) for k, v in comp.items()}
    y, dz = y.astype(np.float64), dz.astype(np.float64)
    loss = lambda: float((ob.compress_forward(y, comp, kind, wl.d_comp) * dz).sum())
    grads = {k: np.zeros_like(v) for k, v in comp.items()}
    dy = ob.compress_backward(y, dz, comp, grads, kind, wl.d_comp)
    assert np.allclose(dy, _fd(loss, y), rtol=1e-5, atol=1e-7)
    for k in comp:
        assert np.allclose(grads[k], _fd(loss, comp[k]), rtol=1e-5, atol=1e-7), k


def test_decompress_backward_matches_finite_differences():
    wl, _, dec, (_, _, z, dx) = _tiny("bottleneck")
    dec = {k: v.astype(np.float64) for k, v in dec.items()}
    z, dx = z.astype(np.float64), dx.astype(np.float64)
    loss = lambda: float((ob.decompress_forward(z, dec) * dx).sum())
    grads = {k: np.zeros_like(v) for k, v in dec.items()}
    dz = ob.decompress_backward(z, dx, dec, grads)
    assert np.allclose(dz, _fd(loss, z), rtol=1e-5, atol=1e-7)
    for k in dec:
        assert np.allclose(grads[k], _fd(loss, dec[k]), rtol=1e-5, atol=1e-7), k


@pytest.mark.parametrize("kind", ["bottleneck", "maxout"])
def test_whole_boundary_against_torch_autograd(kind):
    """receiver(sender(y)) = LN(LN(y) w_c) w_d resp. LN(maxout_k(LN(y))) w_d, re-stated with torch ops."""
    wl, comp, dec, (y, _, _, dx) = _tiny(kind, m=32, c=8, T=9, seed=11)
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    ty, tdx = t(y), torch.tensor(dx, dtype=torch.float64)
    tc = {k: t(v) for k, v in comp.items()}
    td = {k: t(v) for k, v in dec.items()}
    a = torch.nn.functional.layer_norm(ty, (wl.d_model,), tc["ln_g"], tc["ln_b"], wl.ln_eps)
    if kind == "bottleneck":
        z = a @ tc["w_c"].T
    else:
        z = a.reshape(wl.tokens, wl.d_comp, wl.d_model // wl.d_comp).max(dim=-1).values
    x = torch.nn.functional.layer_norm(z, (wl.d_comp,), td["ln_g"], td["ln_b"], wl.ln_eps) @ td["w_d"].T
    (x * tdx).sum().backward()
    # oracle: the two halves chained, the gradient w.r.t. z handed back across the boundary
    zo = ob.compress_forward(y, comp, kind, wl.d_comp)
    xo = ob.decompress_forward(zo, dec)
    gd = {k: np.zeros(v.shape) for k, v in dec.items()}
    gc = {k: np.zeros(v.shape) for k, v in comp.items()}
    dzo = ob.decompress_backward(zo, dx, dec, gd)
    dyo = ob.compress_backward(y, dzo, comp, gc, kind, wl.d_comp)
    assert np.allclose(xo, x.detach().numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dyo, ty.grad.numpy(), rtol=1e-8, atol=1e-11)
    for k in comp:
        assert np.allclose(gc[k], tc[k].grad.numpy(), rtol=1e-8, atol=1e-11), k
    for k in dec:
        assert np.allclose(gd[k], td[k].grad.numpy(), rtol=1e-8, atol=1e-11), k


def test_maxout_known_answers():
    a = np.array([[1.0, 5.0, -2.0, 3.0, 3.0, 0.0], [-1.0, -7.0, 4.0, 4.0, 9.0, 9.5]])
    z, idx = ob.maxout_fwd(a, 2)
    assert np.array_equal(z, [[5.0, 3.0, 3.0], [-1.0, 4.0, 9.5]])
    assert np.array_equal(idx, [[1, 1, 0], [0, 0, 1]])          # ties go to the first feature of the window
    z1, _ = ob.maxout_fwd(a, 1)
    assert np.array_equal(z1, a)                                  # k = 1 is the identity
    z6, _ = ob.maxout_fwd(a, 6)
    assert np.array_equal(z6[:, 0], a.max(axis=1))                # one window = the row maximum
    dz = np.array([[10.0, 20.0, 30.0], [1.0, 2.0, 3.0]])
    da = ob.maxout_bwd(dz, idx, 2)
    assert np.array_equal(da, [[0, 10.0, 0, 20.0, 30.0, 0], [1.0, 0, 2.0, 0, 0, 3.0]])
    assert da.sum() == dz.sum()                                   # gradient mass is routed, not created


def test_maxout_is_permutation_invariant_inside_windows():
    rng = np.random.default_rng(3)
    a = rng.standard_normal((5, 24))
    perm = np.concatenate([w * 4 + rng.permutation(4) for w in range(6)])
    assert np.array_equal(ob.maxout_fwd(a, 4)[0], ob.maxout_fwd(a[:, perm], 4)[0])


def test_bottleneck_with_identity_maps_reduces_to_layernorm():
    """c = m, w_c = w_d = I, unit gains, zero biases: LN(LN(y)) differs from LN(y) only through eps."""
    rng = np.random.default_rng(4)
    m, T = 16, 6
    y = rng.standard_normal((T, m)) * 3.0 + 1.0
    comp = {"ln_g": np.ones(m), "ln_b": np.zeros(m), "w_c": np.eye(m)}
    dec = {"ln_g": np.ones(m), "ln_b": np.zeros(m), "w_d": np.eye(m)}
    x = ob.decompress_forward(ob.compress_forward(y, comp, "bottleneck", m, eps=0.0), dec, eps=0.0)
    ref = (y - y.mean(-1, keepdims=True)) / y.std(-1, keepdims=True)
    assert np.allclose(x, ref, rtol=1e-12, atol=1e-12)


def test_data_transfer_factor_matches_the_appendix_table():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "compression_transfer.txt")) if l[0] != "#"]
    for kind, per_token, rel in rows:
        wl = synth.BOUNDARY_WORKLOADS["%s2_bf16_d4096" % kind]
        comp, dec = synth.make_boundary_params(wl.replace(tokens=2))
        y = synth.make_boundary_inputs(wl.replace(tokens=2))[0]
        z = ob.compress_forward(y, comp, kind, wl.d_comp)
        assert z.shape[1] / y.shape[1] == float(per_token) == float(rel)
        assert ob.decompress_forward(z, dec).shape == y.shape
