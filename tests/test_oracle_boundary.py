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


# ------------------------------------------------------------------ the `store=` argument (maxout decisions on stored values)
def _round_store(a, store):
    """Independent rounding to the storage type (torch's conversions, not the oracle's helpers)."""
    t = torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32)
    if store == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(torch.float64).numpy()


@pytest.mark.parametrize("store", ["f32", "bf16"])
@pytest.mark.parametrize("k", [2, 4, 8])
def test_store_rounding_changes_nothing_but_near_ties(store, k):
    """Rounding is monotone, so deciding on the stored row can never invert an order, only create ties:
      * z(store) is exactly the rounded z(exact);
      * the chosen feature is the first one whose stored value equals the stored window maximum, hence never
        behind the exact winner;
      * wherever the exact runner-up is more than one storage unit below the winner, the choice is the same."""
    m, T = 64 * k, 40
    wl = synth.BoundaryWorkload("st", "f32", "maxout", m, m // k, T, 1.0, seed=90 + k)
    comp, _ = synth.make_boundary_params(wl)
    y, dz, _, _ = synth.make_boundary_inputs(wl)
    z0, c0 = ob.compress_forward(y, comp, "maxout", m // k, keep=True)
    z1, c1 = ob.compress_forward(y, comp, "maxout", m // k, keep=True, store=store)
    a = c0["a"]
    assert np.array_equal(a, c1["a"])                                  # the normalised row itself is untouched
    assert np.array_equal(z1, _round_store(z0, store))
    ar = _round_store(a, store).reshape(T, m // k, k)
    first_max = (ar == ar.max(axis=-1, keepdims=True)).argmax(axis=-1)
    assert np.array_equal(c1["idx"], first_max)
    assert np.all(c1["idx"] <= c0["idx"])
    srt = np.sort(a.reshape(T, m // k, k), axis=-1)
    unit = 2.0 ** (np.floor(np.log2(np.abs(srt).max(axis=-1))) - (7 if store == "bf16" else 23))
    clear = srt[..., -1] - srt[..., -2] > unit
    assert clear.mean() > (0.5 if store == "bf16" else 0.999)
    assert np.array_equal(c0["idx"][clear], c1["idx"][clear])
    # the backward routes by the same choice: with identical idx rows the two gradients agree exactly
    g0 = {q: np.zeros(v.shape) for q, v in comp.items()}
    g1 = {q: np.zeros(v.shape) for q, v in comp.items()}
    dy0 = ob.compress_backward(y, dz, comp, g0, "maxout", m // k)
    dy1 = ob.compress_backward(y, dz, comp, g1, "maxout", m // k, store=store)
    same = (c0["idx"] == c1["idx"]).all(axis=1)
    assert same.any() and np.array_equal(dy0[same], dy1[same])
    if store == "bf16":
        assert not same.all()                                           # bf16 storage does create ties somewhere


def test_store_near_tie_by_hand():
    """Windows built by hand (gain 0, so the normalised row IS the bias row): (1, 1 + 2^-10) is a tie in bf16 -
    the first feature wins - and no tie in fp32 or exact arithmetic; (1 + 2^-30, 1) stays a win of feature 0 in
    every type; (1, 1 + 2^-30) is a tie only once fp32 has rounded it."""
    row = np.array([1.0, 1.0 + 2.0 ** -10, 1.0 + 2.0 ** -30, 1.0, 1.0, 1.0 + 2.0 ** -30, -3.0, -2.0])
    p = {"ln_g": np.zeros(8), "ln_b": row}
    y = np.arange(16, dtype=np.float64).reshape(2, 8) ** 1.5
    dz = np.array([[1.0, 10.0, 100.0, 1000.0], [2.0, 20.0, 200.0, 2000.0]])
    want = {None: [1, 0, 1, 1], "f32": [1, 0, 0, 1], "bf16": [0, 0, 0, 1]}
    for store, idx in want.items():
        z, c = ob.compress_forward(y, p, "maxout", 4, keep=True, store=store)
        assert np.array_equal(c["idx"], np.array([idx, idx])), store
        g = {"ln_g": np.zeros(8), "ln_b": np.zeros(8)}
        ob.compress_backward(y, dz, p, g, "maxout", 4, store=store)
        expect = np.zeros(8)
        for w, i in enumerate(idx):
            expect[2 * w + i] = dz[:, w].sum()                         # d ln_b = column sums of the routed gradient
        assert np.array_equal(g["ln_b"], expect), store
    assert np.array_equal(ob.compress_forward(y, p, "maxout", 4, store="bf16")[0], [1.0, 1.0, 1.0, -2.0])


@pytest.mark.parametrize("kind", ["bottleneck", "maxout"])
def test_fp32_agrees_with_fp64(kind):
    """The full-size GPU parity tests run this oracle in fp32 (dt = np.float32); its fp32 results stay within
    2e-5 (max-normalised) of the fp64 ones at a width and token count where rounding has room to show."""
    m, c, T = 1024, 512, 384
    wl = synth.BoundaryWorkload("p", "f32", kind, m, c, T, 1.0, seed=12)
    comp, dec = synth.make_boundary_params(wl)
    y, dz, z, dx = synth.make_boundary_inputs(wl)
    out = {}
    for dt in (np.float64, np.float32):
        gc = {q: np.zeros(v.shape, dtype=dt) for q, v in comp.items()}
        gd = {q: np.zeros(v.shape, dtype=dt) for q, v in dec.items()}
        # the maxout decision is taken on the same stored values in both precisions, as the parity test does
        st = "f32" if kind == "maxout" else None
        out[dt] = dict(z=ob.compress_forward(y, comp, kind, c, dt=dt, store=st),
                       dy=ob.compress_backward(y, dz, comp, gc, kind, c, dt=dt, store=st),
                       x=ob.decompress_forward(z, dec, dt=dt), dzz=ob.decompress_backward(z, dx, dec, gd, dt=dt),
                       **{"c." + q: v for q, v in gc.items()}, **{"d." + q: v for q, v in gd.items()})
        assert all(v.dtype == dt for v in out[dt].values())
    for q, ref in out[np.float64].items():
        got = out[np.float32][q].astype(np.float64)
        if kind == "maxout" and q in ("dy", "c.ln_g", "c.ln_b"):
            # rows in which fp32 arithmetic moved a stored value across a rounding boundary route differently;
            # they must be rare, and all other rows must agree
            rows = np.abs(out[np.float32]["dy"].astype(np.float64) - out[np.float64]["dy"]).max(axis=1) \
                > 2e-5 * np.abs(out[np.float64]["dy"]).max()
            assert rows.mean() < 0.02
            if q != "dy":
                continue
            got, ref = got[~rows], ref[~rows]
        assert np.max(np.abs(got - ref)) <= 2e-5 * np.max(np.abs(ref)), q
