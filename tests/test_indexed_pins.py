"""Pins of the token-indexed oracle: it must agree with the contiguous-segment oracle applied to the explicitly
sorted batch, and reduce to it for the identity permutation."""
import numpy as np

from oracle import indexed_oracle as io, tlora_oracle as lo


def _case(seed=0):
    rng = np.random.default_rng(seed)
    ranks, tokens = [2, 0, 3], [5, 4, 7]
    off = np.concatenate([[0], np.cumsum(tokens)])
    T, d_in, d_out = off[-1], 6, 5
    X, W, dY = rng.normal(size=(T, d_in)), rng.normal(size=(d_in, d_out)), rng.normal(size=(T, d_out))
    A = [rng.normal(size=(d_in, r)) for r in ranks]
    B = [rng.normal(size=(r, d_out)) for r in ranks]
    return X, W, A, B, [2.0, 1.0, 0.5], off, dY, rng


def test_identity_permutation_is_the_contiguous_layer():
    X, W, A, B, s, off, dY, _ = _case()
    idx = np.arange(X.shape[0])
    Y, dX, dA, dB = io.forward_backward(X, W, A, B, s, off, idx, dY)
    Yr, _ = lo.forward(X, W, A, B, s, off)
    dXr, dAr, dBr, _ = lo.backward(X, W, A, B, s, off, dY)
    np.testing.assert_allclose(Y, Yr, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX, dXr, rtol=1e-12, atol=1e-12)
    for a, b in zip(dA + dB, dAr + dBr):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)


def test_shuffled_batch_equals_sorting_then_contiguous_layer():
    X, W, A, B, s, off, dY, rng = _case(3)
    T = X.shape[0]
    idx = rng.permutation(T)                      # sorted position -> row of the shuffled batch
    Y, dX, dA, dB = io.forward_backward(X, W, A, B, s, off, idx, dY)
    Yr, _ = lo.forward(X[idx], W, A, B, s, off)
    dXr, dAr, dBr, _ = lo.backward(X[idx], W, A, B, s, off, dY[idx])
    np.testing.assert_allclose(Y[idx], Yr, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX[idx], dXr, rtol=1e-12, atol=1e-12)
    for a, b in zip(dA + dB, dAr + dBr):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)
