"""GPU parity of the compression-aware boundary layers (appendix "Compression-Aware Architectures") against the
oracle, through the C ABI.  fp32 within 1e-4, bf16 within 2e-2, max|gpu - oracle| / max|oracle| per output tensor.

Maxout picks one feature per window.  Both sides take that decision on the normalised row as the kernel stores it
(the oracle rounds its own row to the kernel's storage type).  What is left are rows in which a candidate for the
maximum lies so close to a rounding boundary of that type that fp32 versus fp64 arithmetic may round it either
way; those windows are found from the oracle's values alone, and the rows that hold one are checked against the
oracle under every admissible routing (the gradient of such a window lands on one of the features whose stored
value is within one unit of the window's maximum) instead of under the oracle's own routing alone.
"""
import numpy as np
import pytest
import torch

import swarm_synth as synth
from oracle import boundary as ob
from oracle import codec as ocodec
from oracle.stage import layernorm_fwd, layernorm_bwd
from stage_util import max_norm_err

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _dev(a, wl):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(torch.bfloat16) if wl.dtype == "bf16" else t).cuda()


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def run_gpu(wl, comp, dec, y, dz, z, dx):
    import paper_2301_11913_amd as sw
    cfg = sw.BoundaryConfig(wl.d_model, wl.d_comp, wl.kind, wl.tokens, wl.dtype, wl.ln_eps)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    ws = torch.empty(max(sw.swarm_boundary_workspace_bytes(cfg, d, b) for d in (False, True) for b in (False, True)),
                     dtype=torch.uint8, device="cuda")
    cd = {k: _dev(v, wl) for k, v in comp.items()}
    dd = {k: _dev(v, wl) for k, v in dec.items()}
    gc = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in comp.items()}
    gd = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in dec.items()}
    yd, dzd, zd, dxd = (_dev(a, wl) for a in (y, dz, z, dx))
    T, m, c = wl.tokens, wl.d_model, wl.d_comp
    z_out = torch.full((T, c), 7.0, dtype=dt, device="cuda")
    dy = torch.full((T, m), 7.0, dtype=dt, device="cuda")
    x_out = torch.full((T, m), 7.0, dtype=dt, device="cuda")
    dz_out = torch.full((T, c), 7.0, dtype=dt, device="cuda")
    sw.swarm_compress_forward(cfg, cd, yd, z_out, ws)
    sw.swarm_compress_backward(cfg, cd, yd, dzd, dy, gc, ws)
    sw.swarm_decompress_forward(cfg, dd, zd, x_out, ws)
    sw.swarm_decompress_backward(cfg, dd, zd, dxd, dz_out, gd, ws)
    torch.cuda.synchronize()
    return dict(z=_f64(z_out), dy=_f64(dy), x=_f64(x_out), dz=_f64(dz_out),
                gc={k: _f64(v) for k, v in gc.items()}, gd={k: _f64(v) for k, v in gd.items()})


def run_oracle(wl, comp, dec, y, dz, z, dx, dt=np.float64):
    store = wl.dtype if wl.kind == "maxout" else None
    gc = {k: np.zeros(v.shape, dtype=dt) for k, v in comp.items()}
    gd = {k: np.zeros(v.shape, dtype=dt) for k, v in dec.items()}
    out = dict(z=ob.compress_forward(y, comp, wl.kind, wl.d_comp, wl.ln_eps, dt, store=store),
               dy=ob.compress_backward(y, dz, comp, gc, wl.kind, wl.d_comp, wl.ln_eps, dt, store=store),
               x=ob.decompress_forward(z, dec, wl.ln_eps, dt),
               dz=ob.decompress_backward(z, dx, dec, gd, wl.ln_eps, dt), gc=gc, gd=gd)
    return out


def _stored(a, dtype):
    a32 = a.astype(np.float32)
    if dtype == "bf16":
        a32 = ocodec.bf16_bits_to_f32(ocodec.f32_to_bf16_bits(a32))
    return a32.astype(np.float64)


def ambiguous_windows(wl, comp, y):
    """Windows in which the feature the gradient goes to may legitimately differ between fp32 and fp64 arithmetic:
    at least two candidates (stored value within one unit of the window maximum) and one of them within 2e-3
    units of a rounding boundary of the storage type.  Uses oracle values only.  Returns (amb [T, c] bool,
    cand [T, c, k] bool)."""
    a = layernorm_fwd(y.astype(np.float64), comp["ln_g"].astype(np.float64), comp["ln_b"].astype(np.float64),
                      wl.ln_eps)[0]
    mant = 8 if wl.dtype == "bf16" else 24
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(a), 1e-30))) - (mant - 1))
    frac = np.abs(a) / ulp
    near_boundary = np.abs(frac - np.floor(frac) - 0.5) < 2e-3
    k = wl.d_model // wl.d_comp
    st = _stored(a, wl.dtype).reshape(wl.tokens, wl.d_comp, k)
    cand = st >= st.max(axis=-1, keepdims=True) - ulp.reshape(st.shape)
    contested = cand.sum(axis=-1) >= 2                      # a lone maximum wins whichever way it rounds
    return contested & (near_boundary.reshape(st.shape) & cand).any(axis=-1), cand


def check_admissible_routing(wl, comp, y, dz, gpu_dy, amb, cand, idx_ref, bound):
    """Rows with ambiguous windows: the GPU's dy row must equal, within `bound`, the oracle's LayerNorm backward
    of SOME admissible routing - every ambiguous window sending its gradient to one of its candidates (features
    whose stored value is within one storage unit of the window maximum), every other window to the oracle's
    choice.  A wrong routing or a wrong LayerNorm backward on these rows fails: moving one window's gradient to
    another feature changes dy by about |dz| there, an order of magnitude above the bound."""
    import itertools
    k = wl.d_model // wl.d_comp
    g64 = comp["ln_g"].astype(np.float64)
    _, xhat, r = layernorm_fwd(y.astype(np.float64), g64, comp["ln_b"].astype(np.float64), wl.ln_eps)
    worst = 0.0
    for t in np.flatnonzero(amb.any(axis=1)):
        wins = np.flatnonzero(amb[t])
        choices = [np.flatnonzero(cand[t, w]) for w in wins]
        assert np.prod([len(c) for c in choices]) <= 4096, "too many admissible routings to enumerate"
        best = np.inf
        for combo in itertools.product(*choices):
            idx = idx_ref[t:t + 1].copy()
            idx[0, wins] = combo
            da = ob.maxout_bwd(dz[t:t + 1].astype(np.float64), idx, k)
            dy = layernorm_bwd(da, xhat[t:t + 1], r[t:t + 1], g64)[0]
            best = min(best, float(np.max(np.abs(gpu_dy[t] - dy[0]))))
        assert best <= bound, ("row %d: no admissible routing explains the GPU's dy" % t, best, bound)
        worst = max(worst, best)
    return worst


def check(wl, dt=np.float64):
    comp, dec = synth.make_boundary_params(wl)
    y, dz, z, dx = synth.make_boundary_inputs(wl)
    gpu = run_gpu(wl, comp, dec, y, dz, z, dx)
    ref = run_oracle(wl, comp, dec, y, dz, z, dx, dt)
    tol = TOL[wl.dtype]
    errs = {k: max_norm_err(gpu[k], ref[k]) for k in ("z", "x", "dz")}
    if wl.kind == "maxout":
        amb, cand = ambiguous_windows(wl, comp, y)
        risky = amb.any(axis=1)
        assert risky.mean() < 0.5, "the strict comparison must still cover most rows"
        errs["dy"] = max_norm_err(gpu["dy"][~risky], ref["dy"][~risky])
        errs["risky_rows"] = int(risky.sum())
        # rows with an ambiguous window: dy is that of an admissible routing, to the same tolerance
        _, c = ob.compress_forward(y, comp, wl.kind, wl.d_comp, wl.ln_eps, np.float64, keep=True, store=wl.dtype)
        errs["dy_risky"] = check_admissible_routing(wl, comp, y, dz, gpu["dy"], amb, cand, c["idx"],
                                                    tol * float(np.max(np.abs(ref["dy"])))) \
            / float(np.max(np.abs(ref["dy"])))
        # and z, on every row, is the window maximum up to one unit of the storage type plus the LayerNorm's own
        # fp32 arithmetic (absolute, rows are O(1))
        k = wl.d_model // wl.d_comp
        a = layernorm_fwd(y.astype(np.float64), comp["ln_g"].astype(np.float64), comp["ln_b"].astype(np.float64),
                          wl.ln_eps)[0]
        win_max = a.reshape(wl.tokens, wl.d_comp, k).max(axis=-1)
        unit = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(win_max), 1e-30))) - (7 if wl.dtype == "bf16" else 23))
        assert np.all(np.abs(gpu["z"] - win_max) <= unit + 1e-5), "z must be the window maximum up to rounding"
    else:
        errs["dy"] = max_norm_err(gpu["dy"], ref["dy"])
    for k in ref["gc"]:
        errs["c." + k] = max_norm_err(gpu["gc"][k], ref["gc"][k])
    for k in ref["gd"]:
        errs["d." + k] = max_norm_err(gpu["gd"][k], ref["gd"][k])
    print(wl.name, wl.kind, wl.dtype, {k: ("%.2e" % v if isinstance(v, float) else v) for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if isinstance(v, float) and not (v <= tol)}
    assert not bad, bad


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind,m,c,T", [
    ("bottleneck", 256, 128, 150),     # ragged token count
    ("bottleneck", 192, 64, 37),
    ("bottleneck", 1024, 512, 512),    # MFMA tile shapes
    ("maxout", 256, 128, 150),         # k = 2
    ("maxout", 512, 128, 77),          # k = 4
    ("maxout", 512, 64, 33),           # k = 8
    ("maxout", 384, 128, 21),          # k = 3: the one-window-per-thread kernel
    ("maxout", 1024, 512, 512),
    ("maxout", 768, 384, 45),          # widths that leave the last pass of the LayerNorm kernels' lanes partly empty
    ("maxout", 1536, 384, 29),
    ("maxout", 6144, 3072, 19),
    ("bottleneck", 6144, 512, 23),
    # every (row width class of the fused LayerNorm + maxout kernels, window) pair not covered above
    ("maxout", 1024, 256, 40), ("maxout", 1024, 128, 40), ("maxout", 2048, 1024, 24), ("maxout", 2048, 256, 24),
    ("maxout", 4096, 2048, 16), ("maxout", 4096, 1024, 16), ("maxout", 4096, 512, 16), ("maxout", 8192, 2048, 12),
    ("maxout", 8192, 1024, 12),
])
def test_boundary_layers(dtype, kind, m, c, T):
    check(synth.BoundaryWorkload("b", dtype, kind, m, c, T, 1.0 if dtype == "f32" else 1e-2, seed=700 + m + c + T))


@pytest.mark.parametrize("name", ["bottleneck2_bf16_d4096", "maxout2_bf16_d4096"])
def test_boundary_layers_full_size(name):
    """The appendix's setting: compression factor 2 at d_model 4096 on 8192 tokens, as bench.py times it."""
    check(synth.BOUNDARY_WORKLOADS[name], dt=np.float32)


def test_gradients_accumulate_and_calls_are_reproducible():
    import paper_2301_11913_amd as sw
    wl = synth.BoundaryWorkload("acc", "bf16", "bottleneck", 256, 128, 96, 1e-2, seed=31)
    comp, dec = synth.make_boundary_params(wl)
    y, dz, z, dx = synth.make_boundary_inputs(wl)
    one = run_gpu(wl, comp, dec, y, dz, z, dx)
    again = run_gpu(wl, comp, dec, y, dz, z, dx)
    for k in ("z", "dy", "x", "dz"):
        assert np.array_equal(one[k], again[k]), k
    for k in one["gc"]:
        assert np.array_equal(one["gc"][k], again["gc"][k]), k
    # two backward calls into the same buffers give exactly twice one call (x + x is exact)
    cfg = sw.BoundaryConfig(wl.d_model, wl.d_comp, wl.kind, wl.tokens, wl.dtype, wl.ln_eps)
    ws = torch.empty(sw.swarm_boundary_workspace_bytes(cfg, False, True), dtype=torch.uint8, device="cuda")
    cd = {k: _dev(v, wl) for k, v in comp.items()}
    gc = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in comp.items()}
    dy = torch.empty((wl.tokens, wl.d_model), dtype=torch.bfloat16, device="cuda")
    for _ in range(2):
        sw.swarm_compress_backward(cfg, cd, _dev(y, wl), _dev(dz, wl), dy, gc, ws)
    torch.cuda.synchronize()
    for k in gc:
        assert np.array_equal(_f64(gc[k]), 2.0 * one["gc"][k]), k


def test_boundary_composes_with_the_int8_codec():
    """z may additionally travel int8-encoded.  Receiver: the same codes (made by the oracle codec from a synthetic
    z) are decoded on both sides - bit-exact - and decompressed.  Sender: the codes of the GPU's z, decoded, match
    the oracle's z within the bf16 tolerance plus half a quantisation step."""
    import paper_2301_11913_amd as sw
    wl = synth.BoundaryWorkload("codec", "bf16", "bottleneck", 512, 256, 128, 1e-2, seed=77)
    comp, dec = synth.make_boundary_params(wl)
    y, _, z_src, _ = synth.make_boundary_inputs(wl)
    cfg = sw.BoundaryConfig(wl.d_model, wl.d_comp, wl.kind, wl.tokens, wl.dtype, wl.ln_eps)
    ws = torch.empty(max(sw.swarm_boundary_workspace_bytes(cfg, d, False) for d in (False, True)), dtype=torch.uint8,
                     device="cuda")
    shape_z = (wl.tokens, wl.d_comp)
    # receiver
    cz, sz = ocodec.encode(z_src.reshape(-1))
    zr = torch.empty(shape_z, dtype=torch.bfloat16, device="cuda")
    sw.swarm_codec_decode(torch.from_numpy(cz).cuda(), torch.from_numpy(sz).cuda(), zr)
    xt = torch.empty((wl.tokens, wl.d_model), dtype=torch.bfloat16, device="cuda")
    sw.swarm_decompress_forward(cfg, {k: _dev(v, wl) for k, v in dec.items()}, zr, xt, ws)
    torch.cuda.synchronize()
    zdec = ocodec.bf16_bits_to_f32(ocodec.decode(cz, sz, out="bf16")).reshape(shape_z)
    assert np.array_equal(zdec, zr.float().cpu().numpy())
    assert max_norm_err(_f64(xt), ob.decompress_forward(zdec, dec, wl.ln_eps)) <= TOL["bf16"]
    # sender
    zt = torch.empty(shape_z, dtype=torch.bfloat16, device="cuda")
    sw.swarm_compress_forward(cfg, {k: _dev(v, wl) for k, v in comp.items()}, _dev(y, wl), zt, ws)
    n = zt.numel()
    codes = torch.empty(n, dtype=torch.int8, device="cuda")
    scales = torch.empty(n // 64, dtype=torch.float32, device="cuda")
    sw.swarm_codec_encode(zt, codes, scales)
    torch.cuda.synchronize()
    z_ref = ob.compress_forward(y, comp, wl.kind, wl.d_comp, wl.ln_eps)
    got = ocodec.decode(codes.cpu().numpy(), scales.cpu().numpy()).reshape(shape_z).astype(np.float64)
    step = np.repeat(scales.cpu().numpy().astype(np.float64), 64).reshape(shape_z)
    assert np.all(np.abs(got - z_ref) <= TOL["bf16"] * np.max(np.abs(z_ref)) + 0.5 * step + 1e-12)
