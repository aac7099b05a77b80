"""CPU oracle for the first- and last-stage extras of the language model.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (paper_2301_11913_amd/, bench.py's timed region)
imports this module; it exists to check the HIP kernels.

Section 4.3: the first pipeline stage also holds the embedding layer and the last one the language-modelling
head (the appendix "Detailed Performance Comparison" describes that last stage as holding only the vocabulary
projection).  The paper prints no formula for either, so the plain definitions are written out:

    embedding           x[t, :] = E[token[t], :]                      E [V, d]
    head + loss         n = LayerNorm(x; ln_g, ln_b)                  (final LayerNorm of a pre-LN Transformer)
                        logits[t, v] = n[t, :] . W[v, :]              W [V, d], no bias
                        loss = mean_t ( logsumexp_v logits[t, v] - logits[t, target[t]] )

and their gradients (d loss / d logits = (softmax - onehot) / T).  A weight matrix with more than V rows (padding
to a tile multiple) may be passed: rows >= V take no part in the loss and receive zero gradient.

Plain numpy; np.matmul / np.add.at are the only library primitives.  Pins (tests/test_oracle_head.py): central
finite differences, PyTorch's F.embedding / F.layer_norm / F.cross_entropy with autograd, closed forms (uniform
logits give log V, gradient rows of the logits sum to zero, a one-hot-dominant row gives loss -> 0).
"""
from __future__ import annotations

import numpy as np

from oracle.stage import layernorm_fwd, layernorm_bwd


def embedding_forward(tokens, table, dt=np.float64):
    return np.asarray(table, dtype=dt)[np.asarray(tokens)]


def embedding_backward(tokens, dx, grad_table):
    """grad_table [V, d] += scatter of dx [T, d] by token id (repeated ids add up)."""
    np.add.at(grad_table, np.asarray(tokens), np.asarray(dx, dtype=grad_table.dtype))


def head_loss(x, targets, p, vocab, eps=1e-5, dt=np.float64, keep=False):
    """x [T, d], targets [T] int -> mean cross-entropy (and per-token losses / cache when keep)."""
    x = np.asarray(x, dtype=dt)
    n, xhat, r = layernorm_fwd(x, np.asarray(p["ln_g"], dt), np.asarray(p["ln_b"], dt), eps)
    W = np.asarray(p["w_vocab"], dt)
    logits = n @ W[:vocab].T
    m = logits.max(axis=-1, keepdims=True)
    lse = np.log(np.exp(logits - m).sum(axis=-1)) + m[:, 0]
    tok = lse - logits[np.arange(x.shape[0]), np.asarray(targets)]
    loss = tok.mean()
    if keep:
        return loss, tok, dict(n=n, xhat=xhat, r=r, logits=logits, lse=lse)
    return loss


def head_loss_backward(x, targets, p, vocab, grads, eps=1e-5, dt=np.float64):
    """Returns (loss, per-token losses, dx [T, d]); ADDS the parameter gradients into `grads`
    (grads["w_vocab"] has as many rows as p["w_vocab"]; rows >= vocab get nothing)."""
    loss, tok, c = head_loss(x, targets, p, vocab, eps, dt, keep=True)
    T = np.shape(x)[0]
    dlogits = np.exp(c["logits"] - c["lse"][:, None])
    dlogits[np.arange(T), np.asarray(targets)] -= 1.0
    dlogits /= T
    W = np.asarray(p["w_vocab"], dt)
    grads["w_vocab"][:vocab] += dlogits.T @ c["n"]
    dn = dlogits @ W[:vocab]
    dx, dg, db = layernorm_bwd(dn, c["xhat"], c["r"], np.asarray(p["ln_g"], dt))
    grads["ln_g"] += dg
    grads["ln_b"] += db
    return loss, tok, dx
