"""CPU oracle for the parameter update that closes a training step (float64 numpy).

TEST INFRASTRUCTURE ONLY (same rules as oracle.py: imported by tests, smoke and the
benchmark's CPU leg, never by the product path; shares no code with the HIP side).

The paper's core ships "most common first-order stochastic optimization algorithms"
written on tensor operations (Section 4.2 "Optimizers"), and its training-loop listing
ends an iteration with `opt.step(); opt.zeroGrad()` after `loss.backward()`, with gradients
added into the parameters' gradient buffers (the cosine-operator listing's addGrad).
It gives no update formulas, so these are the textbook ones, in the form the common
frameworks use (pinned against torch.optim in the tests):

  SGD   g' = g + wd*p;  buf = mu*buf + g'  (buf starts at 0);  p -= lr*buf   (mu = 0: p -= lr*g')
  Adam  g' = g + wd*p;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2;
        p -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = 1, 2, ...
"""
from __future__ import annotations

import numpy as np


def sgd_step(p, g, buf, *, lr, momentum=0.0, weight_decay=0.0):
    """Returns (p_new, buf_new).  `buf` is the momentum buffer (zeros before the first step)."""
    p, g, buf = (np.asarray(a, np.float64) for a in (p, g, buf))
    gp = g + weight_decay * p
    buf_new = momentum * buf + gp
    return p - lr * buf_new, buf_new


def adam_step(p, g, m, v, *, lr, step, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """Returns (p_new, m_new, v_new).  `step` is 1 for the first update."""
    p, g, m, v = (np.asarray(a, np.float64) for a in (p, g, m, v))
    gp = g + weight_decay * p
    m_new = beta1 * m + (1.0 - beta1) * gp
    v_new = beta2 * v + (1.0 - beta2) * gp * gp
    mhat = m_new / (1.0 - beta1 ** step)
    vhat = v_new / (1.0 - beta2 ** step)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m_new, v_new


def accumulate(grad_old, grad_new):
    """Gradient accumulation (the paper's addGrad): the new gradient is added to the stored one."""
    return np.asarray(grad_old, np.float64) + np.asarray(grad_new, np.float64)
