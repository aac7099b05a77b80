"""Pins for the stage oracle.  CPU only.

Independent references used here: central finite differences (fp64), PyTorch's
own TransformerEncoderLayer + autograd in fp64 (the layer the paper's appendix
"Additional Details for Section 4.1" says it ran), closed-form LayerNorm /
softmax invariants, the causal-mask property, and the structural invariants
of the method (shared == unrolled, accumulation == concatenation).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import stage as osg
import swarm_synth as synth

HERE = os.path.dirname(__file__)

TINY = synth.Workload(name="tiny", dtype="f32", d_model=16, n_heads=2, d_ffn=32, seq=5, batch=2,
                      n_layers=1, n_repeat=1, grad_sigma=1.0, seed=99)


def _tiny(L=1, R=1, scale_w=0.3):
    wl = TINY.replace(n_layers=L, n_repeat=R)
    params = synth.make_params(wl)
    # larger weights than the workloads' 0.02 so every path carries signal in the FD check
    for p in params:
        for k in p:
            if k.startswith("w_") or k.startswith("b_") or k.endswith("_b"):
                p[k] = p[k] * (scale_w / 0.02)
    return wl, params, synth.make_x_in(wl), synth.make_grad_out(wl)


def _loss(params, x, G, wl):
    y = osg.stage_forward(params, x, wl.n_heads, wl.n_repeat, wl.ln_eps, np.float64)
    return float((y * G).sum())


@pytest.mark.parametrize("L,R", [(1, 1), (2, 1), (1, 3), (2, 2)])
def test_finite_differences(L, R):
    wl, params, x, G = _tiny(L, R)
    x = x.astype(np.float64)
    G = G.astype(np.float64)
    params = osg.cast_params(params, np.float64)
    grads = osg.zero_grads(params)
    gin = osg.stage_backward(params, x, G, grads, wl.n_heads, wl.n_repeat, wl.ln_eps)
    eps = 1e-6
    rng = np.random.default_rng(1)
    # every input element
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp = x.copy(); xp[idx] += eps
        xm = x.copy(); xm[idx] -= eps
        fd[idx] = (_loss(params, xp, G, wl) - _loss(params, xm, G, wl)) / (2 * eps)
    assert np.max(np.abs(fd - gin)) <= 1e-6 * max(1.0, np.max(np.abs(gin)))
    # a sample of every parameter tensor of every layer
    for l in range(L):
        for k in osg.PARAM_FIELDS:
            arr = params[l][k]
            flat = rng.choice(arr.size, size=min(6, arr.size), replace=False)
            for f in flat:
                idx = np.unravel_index(f, arr.shape)
                old = arr[idx]
                arr[idx] = old + eps
                lp = _loss(params, x, G, wl)
                arr[idx] = old - eps
                lm = _loss(params, x, G, wl)
                arr[idx] = old
                num = (lp - lm) / (2 * eps)
                ref = grads[l][k][idx]
                assert abs(num - ref) <= 2e-6 * max(1.0, np.max(np.abs(grads[l][k]))), (l, k, idx, num, ref)


def _torch_layer(p, wl, dtype=torch.float64):
    layer = torch.nn.TransformerEncoderLayer(wl.d_model, wl.n_heads, wl.d_ffn, dropout=0.0,
                                             activation="gelu", layer_norm_eps=wl.ln_eps,
                                             batch_first=True, norm_first=True, dtype=dtype)
    with torch.no_grad():
        T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
        layer.norm1.weight.copy_(T(p["ln1_g"])); layer.norm1.bias.copy_(T(p["ln1_b"]))
        layer.self_attn.in_proj_weight.copy_(T(p["w_qkv"])); layer.self_attn.in_proj_bias.copy_(T(p["b_qkv"]))
        layer.self_attn.out_proj.weight.copy_(T(p["w_o"])); layer.self_attn.out_proj.bias.copy_(T(p["b_o"]))
        layer.norm2.weight.copy_(T(p["ln2_g"])); layer.norm2.bias.copy_(T(p["ln2_b"]))
        layer.linear1.weight.copy_(T(p["w_1"])); layer.linear1.bias.copy_(T(p["b_1"]))
        layer.linear2.weight.copy_(T(p["w_2"])); layer.linear2.bias.copy_(T(p["b_2"]))
    return layer


def _torch_names(layer):
    return {"ln1_g": layer.norm1.weight, "ln1_b": layer.norm1.bias,
            "w_qkv": layer.self_attn.in_proj_weight, "b_qkv": layer.self_attn.in_proj_bias,
            "w_o": layer.self_attn.out_proj.weight, "b_o": layer.self_attn.out_proj.bias,
            "ln2_g": layer.norm2.weight, "ln2_b": layer.norm2.bias,
            "w_1": layer.linear1.weight, "b_1": layer.linear1.bias,
            "w_2": layer.linear2.weight, "b_2": layer.linear2.bias}


@pytest.mark.parametrize("shape", [(16, 2, 32, 5, 2, 2, 1), (64, 4, 96, 33, 3, 1, 2), (128, 2, 256, 40, 2, 2, 2)])
def test_against_torch_encoder_layer(shape):
    d, H, f, S, B, L, R = shape
    wl = TINY.replace(d_model=d, n_heads=H, d_ffn=f, seq=S, batch=B, n_layers=L, n_repeat=R)
    params = synth.make_params(wl)
    for p in params:
        for k in p:
            if k[0] in "wb":
                p[k] = p[k] * 5.0
    x, G = synth.make_x_in(wl), synth.make_grad_out(wl)
    layers = [_torch_layer(p, wl) for p in params]
    xt = torch.from_numpy(x.astype(np.float64)).requires_grad_(True)
    mask = torch.triu(torch.full((S, S), float("-inf"), dtype=torch.float64), diagonal=1)
    z = xt
    torch.backends.mha.set_fastpath_enabled(False)
    for layer in layers:
        layer.train()
        for _ in range(R):
            z = layer(z, src_mask=mask)
    z.backward(torch.from_numpy(G.astype(np.float64)))
    y = osg.stage_forward(params, x, H, R, wl.ln_eps, np.float64)
    grads = osg.zero_grads(params)
    gin = osg.stage_backward(params, x, G, grads, H, R, wl.ln_eps)
    assert np.allclose(y, z.detach().numpy(), rtol=1e-10, atol=1e-10)
    assert np.allclose(gin, xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    for l, layer in enumerate(layers):
        for k, t in _torch_names(layer).items():
            ref = t.grad.numpy()
            assert np.allclose(grads[l][k], ref, rtol=1e-9, atol=1e-10 * max(1.0, np.abs(ref).max())), (l, k)


def test_fp32_agrees_with_fp64():
    wl = synth.WORKLOADS["block_f32_d256"].replace(seq=48, batch=2)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    g64 = osg.zero_grads(params, np.float64)
    g32 = osg.zero_grads(params, np.float32)
    y64 = osg.stage_forward(params, x, wl.n_heads, 1, wl.ln_eps, np.float64)
    y32 = osg.stage_forward(params, x, wl.n_heads, 1, wl.ln_eps, np.float32)
    assert y32.dtype == np.float32
    gi64 = osg.stage_backward(params, x, G, g64, wl.n_heads, 1, wl.ln_eps, np.float64)
    gi32 = osg.stage_backward(params, x, G, g32, wl.n_heads, 1, wl.ln_eps, np.float32)
    rel = lambda a, b: np.max(np.abs(a - b)) / np.max(np.abs(b))
    assert rel(y32, y64) < 1e-5 and rel(gi32, gi64) < 1e-5
    for k in osg.PARAM_FIELDS:
        assert g32[0][k].dtype == np.float32
        assert rel(g32[0][k], g64[0][k]) < 1e-5, k


def test_causal_mask():
    wl, params, x, G = _tiny(1, 1)
    y0 = osg.stage_forward(params, x, wl.n_heads)
    j = 3
    x2 = x.copy()
    x2[:, j, :] += 1.0
    y1 = osg.stage_forward(params, x2, wl.n_heads)
    assert np.array_equal(y0[:, :j], y1[:, :j])          # earlier positions bit-identical
    assert not np.allclose(y0[:, j:], y1[:, j:])
    # gradient w.r.t. the last token only comes from the last output position
    Gl = np.zeros_like(G); Gl[:, 0, :] = G[:, 0, :]
    gi = osg.stage_backward(params, x, Gl, osg.zero_grads(params), wl.n_heads)
    assert np.all(gi[:, 1:, :] == 0)


def test_seq_one_attention_is_v():
    q = np.random.default_rng(0).standard_normal((2, 3, 1, 8))
    k = q + 1.0
    v = q * 2.0
    o, p = osg.attention_fwd(q, k, v)
    assert np.array_equal(o, v) and np.all(p == 1.0)


def test_layernorm_and_softmax_invariants():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((7, 48)) * 3 + 1
    g = rng.standard_normal(48); b = rng.standard_normal(48)
    eps = 1e-5
    y, xhat, r = osg.layernorm_fwd(x, g, b, eps)
    v = x.var(axis=-1)
    assert np.allclose(xhat.mean(-1), 0, atol=1e-14)
    assert np.allclose((xhat ** 2).mean(-1), v / (v + eps), rtol=1e-12)
    assert np.allclose(y, torch.nn.functional.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g),
                                                         torch.from_numpy(b), eps).numpy(), rtol=1e-12, atol=1e-12)
    dy = rng.standard_normal((7, 48))
    dx, dg, db = osg.layernorm_bwd(dy, xhat, r, g)
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)             # orthogonal to 1
    # orthogonal to xhat up to the eps term: sum(dx*xhat) = r * sum(t*xhat) * eps/(v+eps)
    t = dy * g
    assert np.allclose((dx * xhat).sum(-1), r[:, 0] * (t * xhat).sum(-1) * eps / (v + eps), rtol=1e-9, atol=1e-14)
    _, xh0, r0 = osg.layernorm_fwd(x, g, b, 0.0)
    dx0, _, _ = osg.layernorm_bwd(dy, xh0, r0, g)
    assert np.allclose((dx0 * xh0).sum(-1), 0, atol=1e-12)    # exactly orthogonal when eps = 0
    q = rng.standard_normal((1, 2, 9, 4)); k = rng.standard_normal((1, 2, 9, 4)); vv = rng.standard_normal((1, 2, 9, 4))
    o, p = osg.attention_fwd(q, k, vv)
    assert np.allclose(p.sum(-1), 1, atol=1e-14)
    assert np.all(np.triu(p[0, 0], 1) == 0)
    do = rng.standard_normal(o.shape)
    dq, dk, dv = osg.attention_bwd(do, q, k, vv, p)
    # rows of dS sum to zero  <=>  shifting all scores of a row changes nothing  <=>  dq . (sum_j p_ij k_j) form
    dp = do @ vv.transpose(0, 1, 3, 2)
    ds = p * (dp - (p * dp).sum(-1, keepdims=True))
    assert np.allclose(ds.sum(-1), 0, atol=1e-13)
    assert np.allclose((p * dp).sum(-1), (do * o).sum(-1), atol=1e-13)


def test_gelu_closed_forms():
    u = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    ref = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u])
    assert np.allclose(osg.gelu(u), ref, rtol=1e-15, atol=0)
    assert osg.gelu(np.zeros(1))[0] == 0 and osg.gelu_grad(np.zeros(1))[0] == 0.5
    h = 1e-6
    assert np.allclose(osg.gelu_grad(u), (osg.gelu(u + h) - osg.gelu(u - h)) / (2 * h), atol=1e-9)
    # x - gelu(x) = gelu(-x) * -1  (symmetry of the normal CDF)
    assert np.allclose(osg.gelu(u) - u, osg.gelu(-u), atol=1e-15)


def test_shared_equals_unrolled():
    wl, params, x, G = _tiny(1, 3)
    unrolled = [dict(params[0]) for _ in range(3)]
    y_s = osg.stage_forward(params, x, wl.n_heads, 3)
    y_u = osg.stage_forward(unrolled, x, wl.n_heads, 1)
    assert np.array_equal(y_s, y_u)
    gs = osg.zero_grads(params); gu = osg.zero_grads(unrolled)
    gi_s = osg.stage_backward(params, x, G, gs, wl.n_heads, 3)
    gi_u = osg.stage_backward(unrolled, x, G, gu, wl.n_heads, 1)
    assert np.array_equal(gi_s, gi_u)
    for k in osg.PARAM_FIELDS:
        tot = gu[0][k] + gu[1][k] + gu[2][k]
        assert np.allclose(gs[0][k], tot, rtol=1e-12, atol=1e-14), k


def test_accumulation_equals_concatenation():
    wl, params, x, G = _tiny(2, 1)
    wl2 = wl.replace(seed=123)
    x2, G2 = synth.make_x_in(wl2), synth.make_grad_out(wl2)
    acc = osg.zero_grads(params)
    gi1 = osg.stage_backward(params, x, G, acc, wl.n_heads)
    gi2 = osg.stage_backward(params, x2, G2, acc, wl.n_heads)       # += on top of the first
    cat = osg.zero_grads(params)
    gic = osg.stage_backward(params, np.concatenate([x, x2]), np.concatenate([G, G2]), cat, wl.n_heads)
    assert np.allclose(np.concatenate([gi1, gi2]), gic, rtol=1e-12, atol=1e-14)
    for l in range(2):
        for k in osg.PARAM_FIELDS:
            assert np.allclose(acc[l][k], cat[l][k], rtol=1e-11, atol=1e-13), (l, k)


def test_table6_parameter_and_flop_counts():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "table6_params_flops.txt")) if not l.startswith("#")]
    for name, d, f, H, layers, n_par, flops in rows:
        wl = TINY.replace(d_model=int(d), d_ffn=int(f), n_heads=int(H))
        shapes = wl.param_shapes()
        weights = sum(int(np.prod(shapes[k])) for k in ("w_qkv", "w_o", "w_1", "w_2"))
        assert weights == 12 * int(d) ** 2
        assert abs(weights - float(n_par)) / float(n_par) < 0.005
        model_flops = 6 * weights * 512 * int(layers)
        assert abs(model_flops - float(flops)) / float(flops) < 0.04


# ------------------------------------------------------------------ rotary + GeGLU block
def _tiny_rg(L=1, R=1):
    wl = TINY.replace(n_layers=L, n_repeat=R, block="rotary_geglu", seed=71)
    params = synth.make_params(wl)
    for p in params:
        for k in p:
            if k[0] in "wb" or k.endswith("_b"):
                p[k] = p[k] * 15.0
    return wl, params, synth.make_x_in(wl), synth.make_grad_out(wl)


@pytest.mark.parametrize("L,R", [(1, 1), (1, 3), (2, 1)])
def test_rotary_geglu_finite_differences(L, R):
    wl, params, x, G = _tiny_rg(L, R)
    x, G = x.astype(np.float64), G.astype(np.float64)
    params = osg.cast_params(params, np.float64)
    kind = "rotary_geglu"
    loss = lambda P, X: float((osg.stage_forward(P, X, wl.n_heads, R, wl.ln_eps, np.float64, kind=kind) * G).sum())
    grads = osg.zero_grads(params)
    gin = osg.stage_backward(params, x, G, grads, wl.n_heads, R, wl.ln_eps, kind=kind)
    eps = 1e-6
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp = x.copy(); xp[idx] += eps
        xm = x.copy(); xm[idx] -= eps
        fd[idx] = (loss(params, xp) - loss(params, xm)) / (2 * eps)
    assert np.max(np.abs(fd - gin)) <= 1e-6 * max(1.0, np.max(np.abs(gin)))
    rng = np.random.default_rng(2)
    for l in range(L):
        for k in osg.PARAM_FIELDS:
            arr = params[l][k]
            for f in rng.choice(arr.size, size=min(6, arr.size), replace=False):
                idx = np.unravel_index(f, arr.shape)
                old = arr[idx]
                arr[idx] = old + eps; lp = loss(params, x)
                arr[idx] = old - eps; lm = loss(params, x)
                arr[idx] = old
                assert abs((lp - lm) / (2 * eps) - grads[l][k][idx]) <= 2e-6 * max(1.0, np.max(np.abs(grads[l][k]))), (l, k)


def test_rotary_geglu_against_torch_autograd():
    """Independent re-statement with PyTorch ops (complex-number rotary, F.gelu, scaled_dot_product-free
    attention) and autograd, fp64."""
    wl = TINY.replace(d_model=64, n_heads=4, d_ffn=96, seq=19, batch=2, n_layers=1, n_repeat=2,
                      block="rotary_geglu", seed=5)
    params, x, G = synth.make_params(wl), synth.make_x_in(wl), synth.make_grad_out(wl)
    for k in params[0]:
        if k[0] in "wb":
            params[0][k] = params[0][k] * 6.0
    P = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in params[0].items()}
    xt = torch.tensor(x.astype(np.float64), requires_grad=True)
    B, S, d, H = wl.batch, wl.seq, wl.d_model, wl.n_heads
    dh, f = d // H, wl.d_ffn
    pos = torch.arange(S, dtype=torch.float64)
    inv = 10000.0 ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    rot = torch.polar(torch.ones(S, dh // 2, dtype=torch.float64), pos[:, None] * inv[None, :])   # e^{i angle}

    def rope(t):                                   # t [B,H,S,dh]
        tc = torch.view_as_complex(t.reshape(B, H, S, dh // 2, 2).contiguous())
        return torch.view_as_real(tc * rot).reshape(B, H, S, dh)

    z = xt
    for _ in range(wl.n_repeat):
        a = torch.nn.functional.layer_norm(z, (d,), P["ln1_g"], P["ln1_b"], wl.ln_eps)
        qkv = a @ P["w_qkv"].T + P["b_qkv"]
        q, k, v = (t.reshape(B, S, H, dh).transpose(1, 2) for t in qkv.split(d, dim=-1))
        q, k = rope(q), rope(k)
        s = q @ k.transpose(-1, -2) / math.sqrt(dh)
        s = s.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf"))
        o = (torch.softmax(s, -1) @ v).transpose(1, 2).reshape(B, S, d)
        h = z + o @ P["w_o"].T + P["b_o"]
        c = torch.nn.functional.layer_norm(h, (d,), P["ln2_g"], P["ln2_b"], wl.ln_eps)
        u = c @ P["w_1"].T + P["b_1"]
        g = torch.nn.functional.gelu(u[..., :f]) * u[..., f:]
        z = h + g @ P["w_2"].T + P["b_2"]
    z.backward(torch.tensor(G.astype(np.float64)))
    kind = "rotary_geglu"
    y = osg.stage_forward(params, x, H, wl.n_repeat, wl.ln_eps, np.float64, kind=kind)
    grads = osg.zero_grads(params)
    gin = osg.stage_backward(params, x, G, grads, H, wl.n_repeat, wl.ln_eps, kind=kind)
    assert np.allclose(y, z.detach().numpy(), rtol=1e-10, atol=1e-10)
    assert np.allclose(gin, xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    for k in osg.PARAM_FIELDS:
        ref = P[k].grad.numpy()
        assert np.allclose(grads[0][k], ref, rtol=1e-9, atol=1e-10 * max(1.0, np.abs(ref).max())), k


def test_rotary_properties():
    rng = np.random.default_rng(8)
    S, dh = 11, 8
    q = rng.standard_normal((1, 1, S, dh)); k = rng.standard_normal((1, 1, S, dh))
    cos, sin = osg.rotary_angles(S, dh, np.float64)
    rq, rk = osg.rotary(q, cos, sin), osg.rotary(k, cos, sin)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1))        # rotations keep norms
    assert np.array_equal(rq[0, 0, 0], q[0, 0, 0])                                       # position 0 is the identity
    assert np.allclose(osg.rotary(rq, cos, sin, inverse=True), q, atol=1e-14)
    # relative-position property: <R_i q, R_j k> depends on i - j only
    q1 = np.broadcast_to(q[:, :, :1], q.shape); k1 = np.broadcast_to(k[:, :, :1], k.shape)
    sc = osg.rotary(q1, cos, sin)[0, 0] @ osg.rotary(k1, cos, sin)[0, 0].T
    for off in range(-3, 4):
        dgl = np.diagonal(sc, off)
        assert np.allclose(dgl, dgl[0], atol=1e-12)
    # first pair rotates by exactly pos radians
    assert np.allclose(cos[:, 0], np.cos(np.arange(S))) and np.allclose(sin[:, 0], np.sin(np.arange(S)))


def test_section43_parameter_count():
    row = [l.split() for l in open(os.path.join(HERE, "golden", "section43_model.txt")) if not l.startswith("#")][0]
    total, stages, d, shared, vocab = float(row[0]), int(row[1]), int(row[2]), int(row[3]), int(row[4])
    wl = synth.WORKLOADS["shared16_rope_geglu_d4096"]
    assert wl.d_model == d and wl.n_repeat == shared and wl.n_layers == 1
    shapes = wl.param_shapes()
    per_stage = sum(int(np.prod(shapes[k])) for k in ("w_qkv", "w_o", "w_1", "w_2"))
    assert per_stage == 4 * d * d + 3 * d * wl.d_ffn
    model = stages * per_stage + vocab * d           # embedding shared with the LM head
    # the paper prints three digits (1.01 B): half a unit of the last digit
    close = lambda n: abs(n - total) <= 0.005e9
    assert close(model)
    # what the printed total excludes: a plain GeLU feed-forward (two d x f matrices), no vocabulary matrix,
    # two untied vocabulary matrices, unshared layers, or another width
    f = wl.d_ffn
    assert not close(stages * (4 * d * d + 2 * d * f) + vocab * d)
    assert not close(stages * per_stage)
    assert not close(stages * per_stage + 2 * vocab * d)
    assert not close(stages * shared * per_stage + vocab * d)
    assert not close(stages * (4 * (d // 2) ** 2 + 3 * (d // 2) * f) + vocab * d)
