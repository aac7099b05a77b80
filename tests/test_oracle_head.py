"""Pins for the embedding / language-modelling-head oracle (oracle/head.py).  CPU only.

Independent references: central finite differences; PyTorch's F.embedding, F.layer_norm, F.cross_entropy with
autograd in fp64; closed forms of the cross-entropy.
"""
import math

import numpy as np
import torch

from oracle import head as oh
import swarm_synth as synth


def _tiny(T=9, d=16, V=11, rows=16, seed=3):
    wl = synth.HeadWorkload("tiny", "f32", d, V, rows, T, seed=seed)
    table, head = synth.make_head_params(wl)
    head["w_vocab"][:V] *= 20.0          # logits of order one, so the softmax is far from uniform
    tokens, targets, x, dxe = synth.make_head_inputs(wl)
    return wl, table.astype(np.float64), {k: v.astype(np.float64) for k, v in head.items()}, tokens, targets, \
        x.astype(np.float64), dxe.astype(np.float64)


def _fd(f, arr, eps=1e-6):
    g = np.zeros_like(arr)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = arr[i]
        arr[i] = old + eps; fp = f()
        arr[i] = old - eps; fm = f()
        arr[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def test_head_backward_matches_finite_differences():
    wl, _, head, _, targets, x, _ = _tiny()
    loss_fn = lambda: float(oh.head_loss(x, targets, head, wl.vocab))
    grads = {k: np.zeros_like(v) for k, v in head.items()}
    loss, tok, dx = oh.head_loss_backward(x, targets, head, wl.vocab, grads)
    assert abs(loss - loss_fn()) < 1e-14 and abs(tok.mean() - loss) < 1e-14
    assert np.allclose(dx, _fd(loss_fn, x), rtol=1e-5, atol=1e-9)
    for k in ("ln_g", "ln_b"):
        assert np.allclose(grads[k], _fd(loss_fn, head[k]), rtol=1e-5, atol=1e-9), k
    gw = _fd(loss_fn, head["w_vocab"])
    assert np.allclose(grads["w_vocab"], gw, rtol=1e-5, atol=1e-9)
    assert np.all(gw[wl.vocab:] == 0.0) and np.all(grads["w_vocab"][wl.vocab:] == 0.0)   # padding rows take no part


def test_embedding_and_head_against_torch():
    wl, table, head, tokens, targets, x, dxe = _tiny(T=12, d=24, V=13, rows=16, seed=8)
    F = torch.nn.functional
    tt = torch.tensor(table, requires_grad=True)
    ids = torch.tensor(tokens, dtype=torch.int64)
    emb = F.embedding(ids, tt)
    assert np.array_equal(emb.detach().numpy(), oh.embedding_forward(tokens, table))
    (emb * torch.tensor(dxe)).sum().backward()
    gt = np.zeros_like(table)
    oh.embedding_backward(tokens, dxe, gt)
    assert np.allclose(gt, tt.grad.numpy(), rtol=1e-12, atol=1e-15)
    assert len(set(tokens.tolist())) < len(tokens)          # the draw has repeated ids: the scatter really adds
    # head
    tx = torch.tensor(x, requires_grad=True)
    tp = {k: torch.tensor(v, requires_grad=True) for k, v in head.items()}
    n = F.layer_norm(tx, (wl.d_model,), tp["ln_g"], tp["ln_b"], wl.ln_eps)
    logits = n @ tp["w_vocab"][:wl.vocab].T
    loss = F.cross_entropy(logits, torch.tensor(targets, dtype=torch.int64), reduction="mean")
    loss.backward()
    grads = {k: np.zeros_like(v) for k, v in head.items()}
    lo, tok, dx = oh.head_loss_backward(x, targets, head, wl.vocab, grads)
    assert abs(lo - loss.item()) < 1e-12
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-13)
    for k in head:
        assert np.allclose(grads[k], tp[k].grad.numpy(), rtol=1e-9, atol=1e-13), k


def test_cross_entropy_closed_forms():
    T, d, V = 5, 8, 7
    x = np.random.default_rng(0).standard_normal((T, d))
    zero_w = {"ln_g": np.ones(d), "ln_b": np.zeros(d), "w_vocab": np.zeros((8, d))}
    targets = np.array([0, 3, 6, 2, 2], dtype=np.int32)
    # all logits equal: loss = log V whatever the targets
    assert abs(oh.head_loss(x, targets, zero_w, V) - math.log(V)) < 1e-14
    # the gradient w.r.t. the logits sums to zero over the vocabulary: dW summed over rows = 0 when n is shared...
    w = {"ln_g": np.ones(d), "ln_b": np.zeros(d), "w_vocab": np.random.default_rng(1).standard_normal((8, d))}
    grads = {k: np.zeros_like(v) for k, v in w.items()}
    oh.head_loss_backward(x, targets, w, V, grads)
    assert np.allclose(grads["w_vocab"][:V].sum(axis=0), 0.0, atol=1e-14)
    # a target whose logit dominates: loss -> 0.  n = LN(x) has norm sqrt(d); make row target = 50 * n
    n = (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, keepdims=True) + 1e-5)
    sharp = {"ln_g": np.ones(d), "ln_b": np.zeros(d), "w_vocab": np.zeros((8, d))}
    sharp["w_vocab"][4] = 50.0 * n[0]
    assert oh.head_loss(x[:1], np.array([4]), sharp, V) < 1e-12
    # and the loss is never negative
    assert oh.head_loss(x, targets, w, V) > 0.0


def test_gpt2_vocabulary_workload_shapes():
    wl = synth.HEAD_WORKLOADS["head_gpt2vocab_bf16_d4096"]
    assert wl.vocab == 50257 and wl.vocab_rows % 256 == 0 and wl.vocab_rows - wl.vocab < 256
    small = wl.replace(d_model=64, tokens=100)
    tokens, targets, x, _ = synth.make_head_inputs(small)
    assert tokens.min() >= 0 and tokens.max() < wl.vocab and targets.max() < wl.vocab


def test_fp32_agrees_with_fp64():
    """The full-size GPU parity test runs this oracle in fp32; its fp32 results stay within 2e-5 (max-normalised;
    the loss relatively) of the fp64 ones on a vocabulary of a few thousand rows."""
    wl = synth.HeadWorkload("p", "f32", 256, 3001, 3008, 96, seed=21)
    table, head = synth.make_head_params(wl)
    head["w_vocab"][:wl.vocab] *= 10.0
    tokens, targets, x, dxe = synth.make_head_inputs(wl)
    out = {}
    for dt in (np.float64, np.float32):
        hp = {k: v.astype(dt) for k, v in head.items()}
        g = {k: np.zeros(v.shape, dtype=dt) for k, v in head.items()}
        res = oh.head_loss_backward(x, targets, hp, wl.vocab, g, wl.ln_eps, dt)
        assert res[2].dtype == dt and res[1].dtype == dt
        out[dt] = (res, g)
    (r64, g64), (r32, g32) = out[np.float64], out[np.float32]
    flat = lambda r: [np.asarray(t, dtype=np.float64) for t in (r if isinstance(r, (tuple, list)) else (r,))]
    for a, b in zip(flat(r32), flat(r64)):
        assert np.max(np.abs(a - b)) <= 2e-5 * max(np.max(np.abs(b)), 1e-30)
    for k in g64:
        assert np.max(np.abs(g32[k].astype(np.float64) - g64[k])) <= 2e-5 * np.max(np.abs(g64[k])), k
