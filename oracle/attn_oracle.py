"""fp64 CPU oracle of the attention half of a decoder layer of the shared super-model.  TEST INFRASTRUCTURE ONLY.

Sec. 3.2 fuses the jobs on one frozen backbone; the backbones of Sec. 4.1 are decoder-only transformers with
rotary position embedding, grouped-query causal self-attention and pre-norm residual blocks.  The paper gives no
formulas for them; these are the standard definitions, written out plainly in float64:

    rope(x)[p, i]          = x[p, i] cos(p w_i) - x[p, i + hd/2] sin(p w_i)            i < hd/2, w_i = base^(-2 i / hd)
    rope(x)[p, i + hd/2]   = x[p, i + hd/2] cos(p w_i) + x[p, i] sin(p w_i)            p = position inside the sequence
    attention, per sequence and query head h (key/value head h // (Hq / Hkv)):
        S = Q K^T / sqrt(hd), keys after the query masked out,  P = softmax(S, axis = keys),  O = P V
    block:  Xn = RMSNorm(X) gamma;  Q, K, V = fused(Xn; W_q / W_k / W_v);  Q, K = rope(Q), rope(K);
            Out = X + fused(attention(Q, K, V); W_o)
    where fused(.) is the multi-LoRA layer of oracle/tlora_oracle.py.

Backward: derivatives of L = sum(dOut * Out) with respect to X and every A_j, B_j (backbone and gamma frozen).
Tokens are rows; `seq_offsets` cuts them into sequences (sequences do not interact).  Tensors are [T, heads * hd],
head-major inside a row.  `store` optionally rounds the tensors the GPU path keeps in memory between kernels.

Pinned by tests/test_attn_pins.py: central finite differences and torch autograd on the CPU (float64), plus closed
forms (a single token attends only to itself; rotary embedding preserves norms and is undone by its transpose).
"""
from __future__ import annotations

import numpy as np

from . import mlp_oracle as mo, tlora_oracle as lo


def _id(a):
    return a


def _angles(n_pos, hd, base):
    w = base ** (-2.0 * np.arange(hd // 2) / hd)
    ang = np.arange(n_pos)[:, None] * w[None, :]
    return np.cos(ang), np.sin(ang)


def rope(x, seq_offsets, n_heads, hd, base, transpose=False):
    """Rotary embedding of every head of x [T, n_heads * hd]; transpose=True applies the inverse rotation (which is
    also the backward of the forward rotation)."""
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    for s in range(len(seq_offsets) - 1):
        lo_, hi = int(seq_offsets[s]), int(seq_offsets[s + 1])
        cos, sin = _angles(hi - lo_, hd, base)
        if transpose:
            sin = -sin
        v = x[lo_:hi].reshape(hi - lo_, n_heads, hd)
        a, b = v[:, :, :hd // 2], v[:, :, hd // 2:]
        r = np.concatenate([a * cos[:, None, :] - b * sin[:, None, :], b * cos[:, None, :] + a * sin[:, None, :]], axis=2)
        out[lo_:hi] = r.reshape(hi - lo_, n_heads * hd)
    return out


def attention(Q, K, V, seq_offsets, n_heads, n_kv, hd):
    """Causal grouped-query attention.  Returns O [T, n_heads * hd] and the softmax matrices (for the backward)."""
    Q, K, V = (np.asarray(a, dtype=np.float64) for a in (Q, K, V))
    O = np.zeros_like(Q)
    probs = {}
    g = n_heads // n_kv
    for s in range(len(seq_offsets) - 1):
        a, b = int(seq_offsets[s]), int(seq_offsets[s + 1])
        n = b - a
        if n == 0:                      # a sequence without tokens contributes nothing
            continue
        mask = np.triu(np.ones((n, n), dtype=bool), k=1)
        for h in range(n_heads):
            q = Q[a:b, h * hd:(h + 1) * hd]
            k = K[a:b, (h // g) * hd:(h // g + 1) * hd]
            v = V[a:b, (h // g) * hd:(h // g + 1) * hd]
            S = q @ k.T / np.sqrt(hd)
            S[mask] = -np.inf
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            O[a:b, h * hd:(h + 1) * hd] = P @ v
            probs[(s, h)] = P
    return O, probs


def attention_lse(Q, K, seq_offsets, n_heads, n_kv, hd):
    """Log-sum-exp of every query's visible scores: lse[t, h] = log(sum over keys <= t of exp(S[t, key])), S = q.k /
    sqrt(hd) -- the logarithm of the softmax denominator (natural logarithm, the textbook statistic)."""
    Q, K = np.asarray(Q, dtype=np.float64), np.asarray(K, dtype=np.float64)
    out = np.zeros((Q.shape[0], n_heads))
    g = n_heads // n_kv
    for s in range(len(seq_offsets) - 1):
        a, b = int(seq_offsets[s]), int(seq_offsets[s + 1])
        for h in range(n_heads):
            S = Q[a:b, h * hd:(h + 1) * hd] @ K[a:b, (h // g) * hd:(h // g + 1) * hd].T / np.sqrt(hd)
            for t in range(b - a):
                row = S[t, :t + 1]
                out[a + t, h] = row.max() + np.log(np.sum(np.exp(row - row.max())))
    return out


def attention_backward(Q, K, V, dO, seq_offsets, n_heads, n_kv, hd):
    Q, K, V, dO = (np.asarray(a, dtype=np.float64) for a in (Q, K, V, dO))
    _, probs = attention(Q, K, V, seq_offsets, n_heads, n_kv, hd)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    g = n_heads // n_kv
    for s in range(len(seq_offsets) - 1):
        a, b = int(seq_offsets[s]), int(seq_offsets[s + 1])
        if a == b:
            continue
        for h in range(n_heads):
            sl, kl = slice(h * hd, (h + 1) * hd), slice((h // g) * hd, (h // g + 1) * hd)
            P = probs[(s, h)]
            do = dO[a:b, sl]
            dV[a:b, kl] += P.T @ do
            dP = do @ V[a:b, kl].T
            dS = P * (dP - np.sum(dP * P, axis=1, keepdims=True))
            dQ[a:b, sl] = dS @ K[a:b, kl] / np.sqrt(hd)
            dK[a:b, kl] += dS.T @ Q[a:b, sl] / np.sqrt(hd)
    return dQ, dK, dV


def block_forward(X, gamma, eps, layers, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, store=_id):
    """layers = {'q': (W, A list, B list), 'k': ..., 'v': ..., 'o': ...}."""
    X = np.asarray(X, dtype=np.float64)
    Xn, rstd = mo.rmsnorm(X, gamma, eps)
    Xn = store(Xn)
    Q, _ = lo.forward(Xn, *layers["q"], scales, offsets)
    K, _ = lo.forward(Xn, *layers["k"], scales, offsets)
    V, _ = lo.forward(Xn, *layers["v"], scales, offsets)
    Q, K, V = store(Q), store(K), store(V)
    Qr, Kr = store(rope(Q, seq_offsets, n_heads, hd, base)), store(rope(K, seq_offsets, n_kv, hd, base))
    O, _ = attention(Qr, Kr, V, seq_offsets, n_heads, n_kv, hd)
    O = store(O)
    D, _ = lo.forward(O, *layers["o"], scales, offsets)
    return X + D, dict(Xn=Xn, rstd=rstd, Qr=Qr, Kr=Kr, V=V, O=O)


def block_backward(X, gamma, eps, layers, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, dOut, store=_id):
    X, dOut, gamma = (np.asarray(a, dtype=np.float64) for a in (X, dOut, gamma))
    _, sv = block_forward(X, gamma, eps, layers, scales, offsets, seq_offsets, n_heads, n_kv, hd, base, store)
    dO, dA_o, dB_o, _ = lo.backward(sv["O"], *layers["o"], scales, offsets, dOut)
    dO = store(dO)
    dQr, dKr, dV = attention_backward(sv["Qr"], sv["Kr"], sv["V"], dO, seq_offsets, n_heads, n_kv, hd)
    dQ = store(rope(store(dQr), seq_offsets, n_heads, hd, base, transpose=True))
    dK = store(rope(store(dKr), seq_offsets, n_kv, hd, base, transpose=True))
    dV = store(dV)
    dXq, dA_q, dB_q, _ = lo.backward(sv["Xn"], *layers["q"], scales, offsets, dQ)
    dXk, dA_k, dB_k, _ = lo.backward(sv["Xn"], *layers["k"], scales, offsets, dK)
    dXv, dA_v, dB_v, _ = lo.backward(sv["Xn"], *layers["v"], scales, offsets, dV)
    dXn = store(dXq) + store(dXk) + store(dXv)
    d = X.shape[1]
    gd = dXn * gamma
    rstd = sv["rstd"]
    dX = dOut + rstd * gd - X * (rstd ** 3) * (np.sum(gd * X, axis=-1, keepdims=True) / d)
    return dX, dict(q=(dA_q, dB_q), k=(dA_k, dB_k), v=(dA_v, dB_v), o=(dA_o, dB_o))
