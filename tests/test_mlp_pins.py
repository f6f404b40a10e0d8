"""Pins of the MLP-block oracle: central finite differences of L = sum(dOut * Out) and torch autograd (CPU,
float64) on small random problems with ragged segments, an empty job and a rank-0 job."""
import numpy as np
import pytest

from oracle import mlp_oracle as mo


def _problem(seed=0, d=6, dff=10, ranks=(2, 0, 3), tokens=(4, 0, 5)):
    rng = np.random.default_rng(seed)
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)])
    X = rng.normal(size=(T, d))
    gamma = 1.0 + 0.1 * rng.normal(size=d)
    layers = {}
    for name, (i, o) in dict(gate=(d, dff), up=(d, dff), down=(dff, d)).items():
        W = rng.normal(size=(i, o)) / np.sqrt(i)
        A = [rng.normal(size=(i, r)) / np.sqrt(i) for r in ranks]
        B = [0.3 * rng.normal(size=(r, o)) for r in ranks]
        layers[name] = (W, A, B)
    scales = [2.0, 1.0, 0.5]
    dOut = rng.normal(size=(T, d))
    return X, gamma, 1e-5, layers, scales, off, dOut


def _loss(X, gamma, eps, layers, scales, off, dOut):
    out, _ = mo.forward(X, gamma, eps, layers, scales, off)
    return float(np.sum(dOut * out))


def test_finite_differences():
    X, gamma, eps, layers, scales, off, dOut = _problem()
    dX, grads = mo.backward(X, gamma, eps, layers, scales, off, dOut)
    h = 1e-6
    rng = np.random.default_rng(1)
    for _ in range(12):                                   # dX entries
        t, i = rng.integers(X.shape[0]), rng.integers(X.shape[1])
        Xp, Xm = X.copy(), X.copy()
        Xp[t, i] += h; Xm[t, i] -= h
        fd = (_loss(Xp, gamma, eps, layers, scales, off, dOut) - _loss(Xm, gamma, eps, layers, scales, off, dOut)) / (2 * h)
        assert abs(fd - dX[t, i]) <= 1e-6 * (1 + abs(fd))
    for name in ("gate", "up", "down"):                   # adapter entries of every layer and job with a rank
        W, A, B = layers[name]
        for j in (0, 2):
            for which, arrs, g in (("A", A, grads[name][0]), ("B", B, grads[name][1])):
                a = arrs[j]
                idx = tuple(rng.integers(s) for s in a.shape)
                keep = a[idx]
                a[idx] = keep + h; fp = _loss(X, gamma, eps, layers, scales, off, dOut)
                a[idx] = keep - h; fm = _loss(X, gamma, eps, layers, scales, off, dOut)
                a[idx] = keep
                fd = (fp - fm) / (2 * h)
                assert abs(fd - g[j][idx]) <= 1e-6 * (1 + abs(fd)), (name, which, j)
    # the job without tokens gets zero gradients, the rank-0 job empty ones
    assert all(np.all(grads[n][0][1] == 0) and grads[n][0][1].shape[1] == 0 for n in grads)


def test_against_torch_autograd_cpu():
    torch = pytest.importorskip("torch")
    X, gamma, eps, layers, scales, off, dOut = _problem(seed=5, d=8, dff=12, ranks=(3, 1, 2), tokens=(3, 6, 2))
    t = lambda a: torch.tensor(a, dtype=torch.float64)
    Xt = t(X).requires_grad_(True)
    params = {n: ([t(a).requires_grad_(True) for a in layers[n][1]], [t(b).requires_grad_(True) for b in layers[n][2]])
              for n in layers}

    def lora(inp, name):
        W = t(layers[name][0])
        rows = []
        for j in range(3):
            x = inp[off[j]:off[j + 1]]
            rows.append(x @ W + scales[j] * (x @ params[name][0][j]) @ params[name][1][j])
        return torch.cat(rows, 0)
    xn = Xt * torch.rsqrt((Xt * Xt).mean(-1, keepdim=True) + eps) * t(gamma)
    z = torch.nn.functional.silu(lora(xn, "gate")) * lora(xn, "up")
    out = Xt + lora(z, "down")
    (out * t(dOut)).sum().backward()
    out_o, _ = mo.forward(X, gamma, eps, layers, scales, off)
    dX_o, grads = mo.backward(X, gamma, eps, layers, scales, off, dOut)
    np.testing.assert_allclose(out.detach().numpy(), out_o, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(Xt.grad.numpy(), dX_o, rtol=1e-10, atol=1e-11)
    for n in layers:
        for j in range(3):
            np.testing.assert_allclose(params[n][0][j].grad.numpy(), grads[n][0][j], rtol=1e-10, atol=1e-11)
            np.testing.assert_allclose(params[n][1][j].grad.numpy(), grads[n][1][j], rtol=1e-10, atol=1e-11)
