"""fp64 CPU oracle of the per-job optimizer step.  TEST INFRASTRUCTURE ONLY (tests and the smoke check).

Sec. 3.2 fixes only that every job fused on the shared backbone keeps its own optimizer state; it names no
optimizer.  The reading taken here is AdamW (Adam with decoupled weight decay, Loshchilov & Hutter) applied to
the adapter tensors A_j, B_j of each job with that job's own hyper-parameters and step count:

    m_t = beta1 m_{t-1} + (1 - beta1) g
    v_t = beta2 v_{t-1} + (1 - beta2) g^2
    mhat = m_t / (1 - beta1^t),   vhat = v_t / (1 - beta2^t)
    w_t = w_{t-1} - lr (mhat / (sqrt(vhat) + eps) + weight_decay w_{t-1})

All arithmetic in float64, elementwise, no fusion.  Pinned by tests/test_adamw_pins.py: closed forms of the first
step (the update is -lr g / (|g| + eps) plus decay), the zero-gradient case (pure decay and geometric moment
decay), a two-step sequence worked by hand, and torch.optim.AdamW on the CPU.
"""
from __future__ import annotations

import numpy as np


def adamw_step(w, g, m, v, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.0):
    """One AdamW step; returns (w_t, m_t, v_t) as float64 arrays.  `step` is t >= 1."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m_t = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v_t = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m_t / (1.0 - beta1 ** step)
    vhat = v_t / (1.0 - beta2 ** step)
    w_t = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w_t, m_t, v_t
