"""fp64 CPU oracle of the MLP half of a decoder layer of the shared super-model.  TEST INFRASTRUCTURE ONLY.

Sec. 3.2: the jobs of a group are fused on one frozen backbone, whose linear layers each carry the jobs' adapters
on the jobs' own tokens.  The backbones the paper trains (Sec. 4.1: 8B-class Llama-3 / Qwen-3 decoders) have a
pre-norm gated MLP; with the three projections replaced by the fused multi-LoRA layer of oracle/tlora_oracle.py it
reads, for the token rows X [T, d]:

    Xn  = X / sqrt(mean(X^2, axis=-1) + eps) * gamma                 (RMSNorm, gamma frozen)
    G   = lora(Xn; W_gate, adapters_gate),   U = lora(Xn; W_up, adapters_up)         [T, d_ff]
    Z   = silu(G) * U,                       silu(g) = g / (1 + exp(-g))
    Out = X + lora(Z; W_down, adapters_down)                                          [T, d]

The backward pass is the derivative of L = sum(dOut * Out) with respect to X and to every A_j, B_j (the backbone
weights and gamma are frozen).  Everything is float64, one numpy operation per line of the definition.
`store` optionally rounds the tensors the GPU path keeps in memory between its kernels (Xn, G, U, Z and the
gradients dZ, dG, dU) to the layer's storage type at the same points -- the decision where to round belongs to
the method's precision, the arithmetic stays fp64.

Pinned by tests/test_mlp_pins.py: central finite differences of L, and torch autograd on the CPU in float64.
"""
from __future__ import annotations

import numpy as np

from . import tlora_oracle as lo


def _id(a):
    return a


def rmsnorm(X, gamma, eps):
    X = np.asarray(X, dtype=np.float64)
    rstd = 1.0 / np.sqrt(np.mean(X * X, axis=-1, keepdims=True) + eps)
    return X * rstd * np.asarray(gamma, dtype=np.float64), rstd


def silu(g):
    return g / (1.0 + np.exp(-g))


def forward(X, gamma, eps, layers, scales, offsets, store=_id):
    """layers = {'gate': (W, A list, B list), 'up': (...), 'down': (...)}.  Returns Out and the saved tensors."""
    X = np.asarray(X, dtype=np.float64)
    Xn, rstd = rmsnorm(X, gamma, eps)
    Xn = store(Xn)
    G, _ = lo.forward(Xn, *layers["gate"], scales, offsets)
    U, _ = lo.forward(Xn, *layers["up"], scales, offsets)
    G, U = store(G), store(U)
    Z = store(silu(G) * U)
    D, _ = lo.forward(Z, *layers["down"], scales, offsets)
    return X + D, dict(Xn=Xn, rstd=rstd, G=G, U=U, Z=Z)


def backward(X, gamma, eps, layers, scales, offsets, dOut, store=_id):
    """dX and {'gate': (dA list, dB list), ...} for L = sum(dOut * Out)."""
    X = np.asarray(X, dtype=np.float64)
    dOut = np.asarray(dOut, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    _, sv = forward(X, gamma, eps, layers, scales, offsets, store)
    dZ, dA_d, dB_d, _ = lo.backward(sv["Z"], *layers["down"], scales, offsets, dOut)
    dZ = store(dZ)
    sig = 1.0 / (1.0 + np.exp(-sv["G"]))
    dU = store(dZ * (sv["G"] * sig))
    dG = store(dZ * sv["U"] * (sig * (1.0 + sv["G"] * (1.0 - sig))))
    dXn_g, dA_g, dB_g, _ = lo.backward(sv["Xn"], *layers["gate"], scales, offsets, dG)
    dXn_u, dA_u, dB_u, _ = lo.backward(sv["Xn"], *layers["up"], scales, offsets, dU)
    dXn = store(dXn_g) + store(dXn_u)
    d = X.shape[1]
    gd = dXn * gamma
    rstd = sv["rstd"]
    dX_norm = rstd * gd - X * (rstd ** 3) * (np.sum(gd * X, axis=-1, keepdims=True) / d)
    return dOut + dX_norm, dict(gate=(dA_g, dB_g), up=(dA_u, dB_u), down=(dA_d, dB_d))
