"""CPU oracle for the LAMB optimiser step.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path imports this module; it exists to check the HIP kernels.

The appendix "Additional Details for Section 4.3" trains with LAMB in the configuration of the optimiser's own
publication, except for the learning rate (1e-3) and beta2 (0.95).  The update of one parameter tensor w (the trust ratio is taken
per tensor, "layer-wise"), for the gradient g accumulated over a global batch:

    g   = grad_scale * grad
    m  <- beta1 m + (1 - beta1) g                  v <- beta2 v + (1 - beta2) g^2
    r   = (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
    u   = r + weight_decay * w
    w  <- w - lr * (||w|| / ||u||) * u             (ratio 1 when either norm is zero)

t = 1, 2, ... is the step number; the norms are Euclidean over the whole tensor.  Plain numpy, fp64.

Pins (tests/test_oracle_lamb.py): PyTorch's own Adam (its moments after several steps, and its step direction,
which LAMB only rescales when weight_decay = 0), and closed forms (||dw|| = lr ||w|| without weight decay;
g = 0 shrinks w by exactly lr; zero weights give ratio 1; grad_scale trades against the gradient's scale).
"""
from __future__ import annotations

import numpy as np


def lamb_step(w, grad, m, v, step, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-6, weight_decay=0.01, grad_scale=1.0,
              dt=np.float64):
    """Returns (w_new, m_new, v_new, trust_ratio); inputs are not modified."""
    w = np.asarray(w, dtype=dt)
    g = np.asarray(grad, dtype=dt) * dt(grad_scale)
    m = dt(beta1) * np.asarray(m, dtype=dt) + dt(1.0 - beta1) * g
    v = dt(beta2) * np.asarray(v, dtype=dt) + dt(1.0 - beta2) * g * g
    r = (m / dt(1.0 - beta1 ** step)) / (np.sqrt(v / dt(1.0 - beta2 ** step)) + dt(eps))
    u = r + dt(weight_decay) * w
    nw, nu = np.sqrt((w * w).sum()), np.sqrt((u * u).sum())
    ratio = nw / nu if (nw > 0 and nu > 0) else dt(1.0)
    return w - dt(lr) * ratio * u, m, v, float(ratio)
