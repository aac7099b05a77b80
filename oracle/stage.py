"""Oracle for one SWARM pipeline stage (TEST INFRASTRUCTURE, not product code).

What a peer of one pipeline stage does to one microbatch (Section 3.2 "SWARM
parallelism"; Section 2.1 "Pipeline parallelism"): forward = apply the stage's
layers to the activations received from the previous stage; backward = take the
gradient w.r.t. the outputs, return the gradient w.r.t. the inputs and
ACCUMULATE the gradients of the parameters.  Stages use activation
checkpointing, so the backward receives only the stage input and recomputes
the forward.  With layer sharing (Sections 2.3 and 4.3) one parameter set is
applied several times in a row and its gradients are summed over the repeats.

The layer is the Transformer layer whose hyper-parameters the appendix
"Additional Details for Section 4.1" lists (d_model, d_FFN, heads); the paper
runs PyTorch's TransformerEncoderLayer there and never writes its equations.
The definition used here: pre-LayerNorm, exact (erf) GeLU, causal
self-attention, biases on all four linear maps, no dropout (the compression
appendix states that dropout is not used), eps = 1e-5 inside the square root,
biased variance, scores scaled by 1/sqrt(d_head).  For a token row x:

    a = LN(x; g1, b1)                     q|k|v = a Wqkv^T + bqkv
    o = concat_h softmax_causal(q_h k_h^T / sqrt(d_h)) v_h
    h = x + o Wo^T + bo
    c = LN(h; g2, b2)                     u = c W1^T + b1,   g = gelu(u)
    y = h + g W2^T + b2

Second block kind, "rotary_geglu" (appendix "Additional Details for Section 4.3": the large-scale model is
the standard Transformer with two changes, rotary position embeddings and GeGLU activations; the paper
gives no formulas, so the cited definitions are used):
  * rotary: in every head, q and k are rotated pairwise, (x_{2i}, x_{2i+1}) by the angle
    pos * 10000^(-2i/d_head), pos = position in the sequence (RoFormer's interleaved form, full head width);
  * GeGLU: u = c W1^T + b1 with W1 [2f, d]; g = gelu(u[:, :f]) * u[:, f:]; y = h + g W2^T + b2 (W2 [d, f]).
Everything else is unchanged.  Pins: finite differences, a PyTorch autograd re-statement, the rotary
relative-position property, and the 1.01 B parameter count of the Section 4.3 model.

Plain numpy; np.matmul is the only library primitive; the arithmetic dtype is
the `dt` argument (float64 for the pins and most parity tests, float32 where
the size demands it).  No blocking, fusion or reordering.

Parity unpinned BY THE PAPER for the block's unstated details (LN placement,
GeLU form, eps, biases): they are fixed by the benchmark description.  The
arithmetic itself is pinned in tests/test_oracle_stage.py by central finite
differences, by PyTorch's own TransformerEncoderLayer + autograd in fp64 (the
layer the paper ran), by closed-form LayerNorm/softmax invariants, by the
causal-mask property, by shared == unrolled, and by microbatch accumulation
== concatenated batch.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf

PARAM_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


# ----------------------------------------------------------------- pieces
def layernorm_fwd(x, gamma, beta, eps):
    """x [T,d].  mu = mean, v = biased variance, r = 1/sqrt(v+eps)."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    v = (xc * xc).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(v + x.dtype.type(eps))
    xhat = xc * r
    return xhat * gamma + beta, xhat, r


def layernorm_bwd(dy, xhat, r, gamma):
    """Returns dx, dgamma, dbeta for y = xhat*gamma + beta."""
    t = dy * gamma
    dx = r * (t - t.mean(axis=-1, keepdims=True)
              - xhat * (t * xhat).mean(axis=-1, keepdims=True))
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def gelu(u):
    return 0.5 * u * (1.0 + erf(u / u.dtype.type(math.sqrt(2.0))))


def gelu_grad(u):
    """d gelu/du = Phi(u) + u phi(u)."""
    cdf = 0.5 * (1.0 + erf(u / u.dtype.type(math.sqrt(2.0))))
    pdf = np.exp(-0.5 * u * u) * u.dtype.type(1.0 / math.sqrt(2.0 * math.pi))
    return cdf + u * pdf


def rotary_angles(S, dh, dt):
    """cos, sin [S, dh/2] of pos * 10000^(-2i/dh)."""
    inv = 10000.0 ** (-np.arange(0, dh, 2, dtype=np.float64) / dh)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(dt), np.sin(ang).astype(dt)


def rotary(t, cos, sin, inverse=False):
    """t [B,H,S,dh]: rotate the pairs (t[..., 2i], t[..., 2i+1]); inverse = rotation by the negative angle."""
    te, to = t[..., 0::2], t[..., 1::2]
    s = -sin if inverse else sin
    out = np.empty_like(t)
    out[..., 0::2] = te * cos - to * s
    out[..., 1::2] = te * s + to * cos
    return out


def _split_heads(t, B, S, H, dh):
    return t.reshape(B, S, H, dh).transpose(0, 2, 1, 3)      # [B,H,S,dh]


def _merge_heads(t, B, S, H, dh):
    return t.transpose(0, 2, 1, 3).reshape(B * S, H * dh)


def attention_fwd(q, k, v):
    """q,k,v [B,H,S,dh]; causal softmax(q k^T / sqrt(dh)) v.  Returns o, p."""
    S, dh = q.shape[2], q.shape[3]
    s = np.matmul(q, k.transpose(0, 1, 3, 2)) * q.dtype.type(1.0 / math.sqrt(dh))
    mask = np.tril(np.ones((S, S), dtype=bool))
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.where(mask, np.exp(s - m), 0.0).astype(q.dtype)
    p = e / e.sum(axis=-1, keepdims=True)
    return np.matmul(p, v), p


def attention_bwd(do, q, k, v, p):
    dh = q.shape[3]
    scale = q.dtype.type(1.0 / math.sqrt(dh))
    dv = np.matmul(p.transpose(0, 1, 3, 2), do)
    dp = np.matmul(do, v.transpose(0, 1, 3, 2))
    delta = (p * dp).sum(axis=-1, keepdims=True)
    ds = p * (dp - delta)
    dq = np.matmul(ds, k) * scale
    dk = np.matmul(ds.transpose(0, 1, 3, 2), q) * scale
    return dq, dk, dv


# ----------------------------------------------------------------- block
def block_forward(x, p, n_heads, eps, B, S, kind="gelu"):
    """x [T,d] -> (y [T,d], cache of intermediates)."""
    T, d = x.shape
    dh = d // n_heads
    a, xh1, r1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = a @ p["w_qkv"].T + p["b_qkv"]
    q = _split_heads(qkv[:, :d], B, S, n_heads, dh)
    k = _split_heads(qkv[:, d:2 * d], B, S, n_heads, dh)
    v = _split_heads(qkv[:, 2 * d:], B, S, n_heads, dh)
    rope = None
    if kind == "rotary_geglu":
        rope = rotary_angles(S, dh, x.dtype)
        q, k = rotary(q, *rope), rotary(k, *rope)
    o4, prob = attention_fwd(q, k, v)
    o = _merge_heads(o4, B, S, n_heads, dh)
    h = x + o @ p["w_o"].T + p["b_o"]
    c, xh2, r2 = layernorm_fwd(h, p["ln2_g"], p["ln2_b"], eps)
    u = c @ p["w_1"].T + p["b_1"]
    if kind == "rotary_geglu":
        f = u.shape[1] // 2
        g = gelu(u[:, :f]) * u[:, f:]
    else:
        g = gelu(u)
    y = h + g @ p["w_2"].T + p["b_2"]
    cache = dict(xh1=xh1, r1=r1, a=a, q=q, k=k, v=v, prob=prob, o=o,
                 xh2=xh2, r2=r2, c=c, u=u, g=g, rope=rope)
    return y, cache


def block_backward(dy, p, cache, grads, n_heads, B, S, kind="gelu"):
    """dy [T,d] -> dx [T,d]; parameter gradients are ADDED into `grads`."""
    T, d = dy.shape
    dh = d // n_heads
    # y = h + g W2^T + b2
    grads["w_2"] += dy.T @ cache["g"]
    grads["b_2"] += dy.sum(axis=0)
    dg = dy @ p["w_2"]
    if kind == "rotary_geglu":
        u = cache["u"]
        f = u.shape[1] // 2
        du = np.concatenate([dg * u[:, f:] * gelu_grad(u[:, :f]), dg * gelu(u[:, :f])], axis=1)
    else:
        du = dg * gelu_grad(cache["u"])
    grads["w_1"] += du.T @ cache["c"]
    grads["b_1"] += du.sum(axis=0)
    dc = du @ p["w_1"]
    dh_ln, dg2, db2 = layernorm_bwd(dc, cache["xh2"], cache["r2"], p["ln2_g"])
    grads["ln2_g"] += dg2
    grads["ln2_b"] += db2
    dhid = dy + dh_ln
    # h = x + o Wo^T + bo
    grads["w_o"] += dhid.T @ cache["o"]
    grads["b_o"] += dhid.sum(axis=0)
    do = dhid @ p["w_o"]
    do4 = _split_heads(do, B, S, n_heads, dh)
    dq, dk, dv = attention_bwd(do4, cache["q"], cache["k"], cache["v"], cache["prob"])
    if kind == "rotary_geglu":          # q, k in the cache are the rotated ones; undo the rotation on their gradients
        dq, dk = rotary(dq, *cache["rope"], inverse=True), rotary(dk, *cache["rope"], inverse=True)
    dqkv = np.concatenate([_merge_heads(dq, B, S, n_heads, dh),
                           _merge_heads(dk, B, S, n_heads, dh),
                           _merge_heads(dv, B, S, n_heads, dh)], axis=1)
    grads["w_qkv"] += dqkv.T @ cache["a"]
    grads["b_qkv"] += dqkv.sum(axis=0)
    da = dqkv @ p["w_qkv"]
    dx_ln, dg1, db1 = layernorm_bwd(da, cache["xh1"], cache["r1"], p["ln1_g"])
    grads["ln1_g"] += dg1
    grads["ln1_b"] += db1
    return dhid + dx_ln


# ----------------------------------------------------------------- stage
def cast_params(params, dt):
    return [{k: np.asarray(p[k], dtype=dt) for k in PARAM_FIELDS} for p in params]


def zero_grads(params, dt=np.float64):
    return [{k: np.zeros(np.shape(p[k]), dtype=dt) for k in PARAM_FIELDS} for p in params]


def stage_forward(params, x_in, n_heads, n_repeat=1, eps=1e-5, dt=np.float64, keep=False, kind="gelu"):
    """x_in [B,S,d] -> x_out [B,S,d]: each of the L parameter sets applied n_repeat times in a row."""
    B, S, d = x_in.shape
    P = cast_params(params, dt)
    z = np.asarray(x_in, dtype=dt).reshape(B * S, d)
    caches = []
    for p in P:
        for _ in range(n_repeat):
            z, cache = block_forward(z, p, n_heads, eps, B, S, kind)
            if keep:
                caches.append(cache)
    out = z.reshape(B, S, d)
    return (out, caches) if keep else out


def stage_backward(params, x_in, grad_out, grad_params, n_heads, n_repeat=1, eps=1e-5,
                   dt=np.float64, kind="gelu"):
    """Checkpointed backward: recompute the forward from x_in, then walk the L*R block
    applications in reverse.  Returns grad_in [B,S,d]; `grad_params` (list of L dicts)
    is accumulated into (+=), a shared set receiving the sum over its repeats."""
    B, S, d = x_in.shape
    P = cast_params(params, dt)
    _, caches = stage_forward(params, x_in, n_heads, n_repeat, eps, dt, keep=True, kind=kind)
    dz = np.asarray(grad_out, dtype=dt).reshape(B * S, d)
    idx = len(caches)
    for l in reversed(range(len(P))):
        for _ in range(n_repeat):
            idx -= 1
            dz = block_backward(dz, P[l], caches[idx], grad_params[l], n_heads, B, S, kind)
            caches[idx] = None
    return dz.reshape(B, S, d)
