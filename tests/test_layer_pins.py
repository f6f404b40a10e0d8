"""Pin of the decoder-layer oracle (attention half then MLP half): central finite differences of the scalar loss
through the whole layer, with respect to the input and to adapters of all seven projections."""
import numpy as np

from oracle import layer_oracle as ly


def _problem(seed=0):
    rng = np.random.default_rng(seed)
    d, dff, Hq, Hkv, hd = 8, 12, 4, 2, 4
    ranks, tokens = (2, 0, 3), (5, 3, 6)
    off = np.concatenate([[0], np.cumsum(tokens)])
    seq = [0, 5, 8, 10, 14]
    T = off[-1]

    def layers(shapes):
        return {n: (rng.normal(size=(i, o)) / np.sqrt(i), [rng.normal(size=(i, r)) / np.sqrt(i) for r in ranks],
                    [0.3 * rng.normal(size=(r, o)) for r in ranks]) for n, (i, o) in shapes.items()}
    attn = (1.0 + 0.1 * rng.normal(size=d), 1e-5, layers(dict(q=(d, Hq * hd), k=(d, Hkv * hd), v=(d, Hkv * hd), o=(Hq * hd, d))))
    mlp = (1.0 + 0.1 * rng.normal(size=d), 1e-5, layers(dict(gate=(d, dff), up=(d, dff), down=(dff, d))))
    return rng.normal(size=(T, d)), attn, mlp, [2.0, 1.0, 0.5], off, seq, Hq, Hkv, hd, 100.0, rng.normal(size=(T, d))


def test_layer_finite_differences():
    X, attn, mlp, scales, off, seq, Hq, Hkv, hd, base, dOut = _problem()
    args = (attn, mlp, scales, off, seq, Hq, Hkv, hd, base)
    loss = lambda Xv: float(np.sum(dOut * ly.forward(Xv, *args)[0]))
    dX, grads = ly.backward(X, *args, dOut)
    assert set(grads) == {"q", "k", "v", "o", "gate", "up", "down"}
    rng = np.random.default_rng(1)
    h = 1e-6
    for _ in range(10):
        t, i = rng.integers(X.shape[0]), rng.integers(X.shape[1])
        Xp, Xm = X.copy(), X.copy()
        Xp[t, i] += h; Xm[t, i] -= h
        fd = (loss(Xp) - loss(Xm)) / (2 * h)
        assert abs(fd - dX[t, i]) <= 2e-6 * (1 + abs(fd))
    for half in (attn, mlp):
        for name in half[2]:
            for j in (0, 2):
                for k in (1, 2):
                    a = half[2][name][k][j]
                    idx = tuple(rng.integers(s) for s in a.shape)
                    keep = a[idx]
                    a[idx] = keep + h; fp = loss(X)
                    a[idx] = keep - h; fm = loss(X)
                    a[idx] = keep
                    fd = (fp - fm) / (2 * h)
                    assert abs(fd - grads[name][k - 1][j][idx]) <= 2e-6 * (1 + abs(fd)), (name, k, j)


def test_layer_with_silent_mlp_is_the_attention_block():
    # zero down-projection (backbone and adapters): the MLP half adds nothing, Out = H
    X, attn, mlp, scales, off, seq, Hq, Hkv, hd, base, _ = _problem(3)
    W, A, B = mlp[2]["down"]
    mlp[2]["down"] = (np.zeros_like(W), A, [np.zeros_like(b) for b in B])
    Out, H = ly.forward(X, attn, mlp, scales, off, seq, Hq, Hkv, hd, base)
    np.testing.assert_array_equal(Out, H)
