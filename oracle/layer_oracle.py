"""fp64 CPU oracle of one decoder layer of the shared super-model.  TEST INFRASTRUCTURE ONLY.

Sec. 3.2: the jobs of a group run as one model on one frozen backbone; the unit the backbone repeats is the
decoder layer (Sec. 4.1's 8B-class decoders): the attention half followed by the MLP half, each pre-norm and
residual, all seven projections being fused multi-LoRA layers:

    H   = attention_block(X)           (oracle/attn_oracle.py)
    Out = mlp_block(H)                 (oracle/mlp_oracle.py)

Backward: derivatives of L = sum(dOut * Out) with respect to X and every A_j, B_j of the seven projections, by the
chain rule through H.  `store` rounds what the GPU path keeps in memory (H, dH and the halves' own tensors).

Pinned by tests/test_layer_pins.py: central finite differences of L through the whole layer.
"""
from __future__ import annotations

import numpy as np

from . import attn_oracle as ao, mlp_oracle as mo


def _id(a):
    return a


def forward(X, attn, mlp, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, store=_id):
    """attn = (gamma, eps, {'q','k','v','o': (W, A list, B list)}),  mlp = (gamma, eps, {'gate','up','down': ...})."""
    H, _ = ao.block_forward(X, attn[0], attn[1], attn[2], scales, offsets, seq_offsets, n_heads, n_kv, hd, base, store)
    H = store(H)
    Out, _ = mo.forward(H, mlp[0], mlp[1], mlp[2], scales, offsets, store)
    return Out, H


def backward(X, attn, mlp, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, dOut, store=_id):
    """dX and the gradients {'q': (dA list, dB list), ..., 'down': (...)}."""
    _, H = forward(X, attn, mlp, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, store)
    dH, g_mlp = mo.backward(H, mlp[0], mlp[1], mlp[2], scales, offsets, dOut, store)
    dH = store(dH)
    dX, g_attn = ao.block_backward(X, attn[0], attn[1], attn[2], scales, offsets, seq_offsets, n_heads, n_kv, hd, base,
                                   dH, store)
    grads = dict(g_attn)
    grads.update(g_mlp)
    return dX, grads
