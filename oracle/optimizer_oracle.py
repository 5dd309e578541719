"""CPU oracle for the optimizer-step instruction of the pipeline (paper, Table 2: "OS", one of the
three runtime-control opcodes; Sec. 3 notes that the BF and BE parameter gradients are summed before
it).  TEST INFRASTRUCTURE ONLY; float64 numpy; shares no code with the library's kernel.

Reading: the paper names no optimizer.  This build takes AdamW (Adam moments with bias correction,
weight decay decoupled from the gradient), the usual choice for the models the paper trains, written
out from its definition:

    g   = grad_scale * grad
    m  <- beta1 m + (1 - beta1) g
    v  <- beta2 v + (1 - beta2) g^2
    theta <- theta - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * theta )

with t = 1 for the first step.  Pins (tests/test_oracle_optimizer.py): torch.optim.AdamW over several
steps (library routine), the first step's closed form lr * g / (|g| + eps), zero gradient leaving only
the decay, and the constant-gradient fixed point m_hat = g, v_hat = g^2 at every t."""
from __future__ import annotations

from typing import Tuple

import numpy as np


def adamw_step(theta: np.ndarray, grad: np.ndarray, m: np.ndarray, v: np.ndarray, t: int, lr: float,
               beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.0,
               grad_scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One update; returns the new (theta, m, v) as float64 arrays (inputs untouched)."""
    assert t >= 1
    theta = np.asarray(theta, dtype=np.float64)
    g = grad_scale * np.asarray(grad, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    theta = theta - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * theta)
    return theta, m, v
