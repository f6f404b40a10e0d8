"""Pins of the attention oracle (rotary embedding, causal grouped-query attention, the pre-norm attention block over
fused multi-LoRA projections): closed forms, central finite differences, torch autograd on the CPU in float64."""
import numpy as np
import pytest

from oracle import attn_oracle as ao


def test_rope_closed_forms():
    rng = np.random.default_rng(0)
    seq = [0, 5, 5, 12]
    x = rng.normal(size=(12, 3 * 8))
    r = ao.rope(x, seq, 3, 8, 10000.0)
    # position 0 of every sequence is not rotated; norms of every (i, i + hd/2) pair are preserved
    np.testing.assert_allclose(r[[0, 5]], x[[0, 5]], rtol=0, atol=1e-15)
    xv, rv = x.reshape(12, 3, 2, 4), r.reshape(12, 3, 2, 4)
    np.testing.assert_allclose((xv ** 2).sum(axis=2), (rv ** 2).sum(axis=2), rtol=1e-12)
    # the transpose undoes it, and one explicit entry: position 3, pair 1 of head 0, w = 10000^(-2/8)
    np.testing.assert_allclose(ao.rope(r, seq, 3, 8, 10000.0, transpose=True), x, rtol=1e-12, atol=1e-14)
    w = 10000.0 ** (-2.0 / 8)
    assert abs(r[3, 1] - (x[3, 1] * np.cos(3 * w) - x[3, 5] * np.sin(3 * w))) < 1e-14
    assert abs(r[3, 5] - (x[3, 5] * np.cos(3 * w) + x[3, 1] * np.sin(3 * w))) < 1e-14


def test_attention_closed_forms():
    rng = np.random.default_rng(1)
    Q, K, V = rng.normal(size=(6, 4 * 8)), rng.normal(size=(6, 2 * 8)), rng.normal(size=(6, 2 * 8))
    O, _ = ao.attention(Q, K, V, [0, 1, 6], 4, 2, 8)
    # the first token of a sequence attends to itself only: its output is its own value row (per kv head)
    for h in range(4):
        np.testing.assert_allclose(O[0, h * 8:(h + 1) * 8], V[0, (h // 2) * 8:(h // 2 + 1) * 8], rtol=1e-14)
        np.testing.assert_allclose(O[1, h * 8:(h + 1) * 8], V[1, (h // 2) * 8:(h // 2 + 1) * 8], rtol=1e-14)
    # zero queries give uniform weights over the visible keys: the running mean of the values
    O0, _ = ao.attention(np.zeros_like(Q), K, V, [0, 6], 4, 2, 8)
    np.testing.assert_allclose(O0[:, :8], np.cumsum(V[:, :8], axis=0) / np.arange(1, 7)[:, None], rtol=1e-13)


def test_lse_matches_library_logsumexp_and_probabilities():
    from scipy.special import logsumexp
    rng = np.random.default_rng(2)
    seq, Hq, Hkv, hd = [0, 3, 3, 9], 4, 2, 8
    Q, K, V = rng.normal(size=(9, Hq * hd)), rng.normal(size=(9, Hkv * hd)), rng.normal(size=(9, Hkv * hd))
    lse = ao.attention_lse(Q, K, seq, Hq, Hkv, hd)
    _, probs = ao.attention(Q, K, V, seq, Hq, Hkv, hd)
    for s, (a, b) in enumerate(zip(seq[:-1], seq[1:])):
        for h in range(Hq):
            for t in range(a, b):
                scores = np.array([Q[t, h * hd:(h + 1) * hd] @ K[u, (h // 2) * hd:(h // 2 + 1) * hd] for u in range(a, t + 1)])
                scores /= np.sqrt(hd)
                assert abs(lse[t, h] - logsumexp(scores)) < 1e-12
                # exp(score - lse) reproduces the probabilities of the attention oracle
                np.testing.assert_allclose(np.exp(scores - lse[t, h]), probs[(s, h)][t - a, :t - a + 1],
                                           rtol=1e-12)


def _block_problem(seed=0):
    rng = np.random.default_rng(seed)
    d, Hq, Hkv, hd = 8, 4, 2, 4
    ranks, tokens = (2, 0, 3), (5, 3, 6)
    off = np.concatenate([[0], np.cumsum(tokens)])
    seq = [0, 2, 5, 8, 14]
    T = off[-1]
    X = rng.normal(size=(T, d))
    gamma = 1.0 + 0.1 * rng.normal(size=d)
    layers = {}
    for name, (i, o) in dict(q=(d, Hq * hd), k=(d, Hkv * hd), v=(d, Hkv * hd), o=(Hq * hd, d)).items():
        layers[name] = (rng.normal(size=(i, o)) / np.sqrt(i), [rng.normal(size=(i, r)) / np.sqrt(i) for r in ranks],
                        [0.3 * rng.normal(size=(r, o)) for r in ranks])
    return X, gamma, 1e-5, layers, [2.0, 1.0, 0.5], off, seq, Hq, Hkv, hd, 100.0, rng.normal(size=(T, d))


def test_block_finite_differences():
    X, gamma, eps, layers, scales, off, seq, Hq, Hkv, hd, base, dOut = _block_problem()
    args = (gamma, eps, layers, scales, off, seq, Hq, Hkv, hd, base)
    loss = lambda Xv: float(np.sum(dOut * ao.block_forward(Xv, *args)[0]))
    dX, grads = ao.block_backward(X, *args, dOut)
    rng = np.random.default_rng(1)
    h = 1e-6
    for _ in range(10):
        t, i = rng.integers(X.shape[0]), rng.integers(X.shape[1])
        Xp, Xm = X.copy(), X.copy()
        Xp[t, i] += h; Xm[t, i] -= h
        fd = (loss(Xp) - loss(Xm)) / (2 * h)
        assert abs(fd - dX[t, i]) <= 2e-6 * (1 + abs(fd))
    for name in layers:
        for j in (0, 2):
            for k, g in ((1, grads[name][0]), (2, grads[name][1])):
                a = layers[name][k][j]
                idx = tuple(rng.integers(s) for s in a.shape)
                keep = a[idx]
                a[idx] = keep + h; fp = loss(X)
                a[idx] = keep - h; fm = loss(X)
                a[idx] = keep
                fd = (fp - fm) / (2 * h)
                assert abs(fd - g[j][idx]) <= 2e-6 * (1 + abs(fd)), (name, k, j)


def test_block_against_torch_autograd_cpu():
    torch = pytest.importorskip("torch")
    X, gamma, eps, layers, scales, off, seq, Hq, Hkv, hd, base, dOut = _block_problem(4)
    t = lambda a: torch.tensor(a, dtype=torch.float64)
    Xt = t(X).requires_grad_(True)
    params = {n: ([t(a).requires_grad_(True) for a in layers[n][1]], [t(b).requires_grad_(True) for b in layers[n][2]])
              for n in layers}

    def lora(inp, name):
        W = t(layers[name][0])
        return torch.cat([inp[off[j]:off[j + 1]] @ W + scales[j] * (inp[off[j]:off[j + 1]] @ params[name][0][j]) @ params[name][1][j]
                          for j in range(3)], 0)

    def rope_t(x, H):
        outs = []
        for s in range(len(seq) - 1):
            n = seq[s + 1] - seq[s]
            w = base ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd)
            ang = torch.arange(n, dtype=torch.float64)[:, None] * w[None, :]
            v = x[seq[s]:seq[s + 1]].reshape(n, H, hd)
            a, b = v[..., :hd // 2], v[..., hd // 2:]
            c, s_ = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
            outs.append(torch.cat([a * c - b * s_, b * c + a * s_], -1).reshape(n, H * hd))
        return torch.cat(outs, 0)
    xn = Xt * torch.rsqrt((Xt * Xt).mean(-1, keepdim=True) + eps) * t(gamma)
    q, k, v = rope_t(lora(xn, "q"), Hq), rope_t(lora(xn, "k"), Hkv), lora(xn, "v")
    outs = []
    for s in range(len(seq) - 1):
        n = seq[s + 1] - seq[s]
        qs = q[seq[s]:seq[s + 1]].reshape(n, Hq, hd).transpose(0, 1)
        ks = k[seq[s]:seq[s + 1]].reshape(n, Hkv, hd).transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
        vs = v[seq[s]:seq[s + 1]].reshape(n, Hkv, hd).transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
        o = torch.nn.functional.scaled_dot_product_attention(qs, ks, vs, is_causal=True)
        outs.append(o.transpose(0, 1).reshape(n, Hq * hd))
    out = Xt + lora(torch.cat(outs, 0), "o")
    (out * t(dOut)).sum().backward()
    args = (gamma, eps, layers, scales, off, seq, Hq, Hkv, hd, base)
    out_o, _ = ao.block_forward(X, *args)
    dX_o, grads = ao.block_backward(X, *args, dOut)
    np.testing.assert_allclose(out.detach().numpy(), out_o, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(Xt.grad.numpy(), dX_o, rtol=1e-9, atol=1e-10)
    for n in layers:
        for j in range(3):
            np.testing.assert_allclose(params[n][0][j].grad.numpy(), grads[n][0][j], rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(params[n][1][j].grad.numpy(), grads[n][1][j], rtol=1e-9, atol=1e-10)
