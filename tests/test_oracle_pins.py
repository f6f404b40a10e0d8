"""Pins for the fp64 oracle: every check compares it with something that does not come from the
oracle itself -- a hand-worked example, pure-Python triple loops, finite differences of the loss,
the dense-weight identity, special cases and structural invariants (Sec. 2, Sec. 3.2, Sec. 3.3)."""
import json
import os

import numpy as np
import pytest

from oracle import tlora_oracle as orc
from paper_2602_07263_amd import workloads as wk

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny(seed=0, d_in=5, d_out=7, ranks=(1, 3), tokens=(2, 3), scales=(2.0, 0.75)):
    rng = np.random.default_rng(seed)
    T = sum(tokens)
    X = rng.standard_normal((T, d_in))
    W = rng.standard_normal((d_in, d_out))
    dY = rng.standard_normal((T, d_out))
    A = [rng.standard_normal((d_in, r)) for r in ranks]
    B = [rng.standard_normal((r, d_out)) for r in ranks]
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    return X, W, A, B, list(scales), off, dY


# -- 1. hand-worked example -----------------------------------------------------------------------
def test_hand_worked_example():
    with open(os.path.join(GOLDEN, "hand_2x2_rank1.json")) as f:
        g = json.load(f)
    X, W, A, B = (np.array(g[k]) for k in ("X", "W", "A", "B"))
    off = np.array([0, 1])
    Y, S = orc.forward(X, W, [A], [B], [g["scale"]], off)
    assert np.array_equal(S[0], np.array(g["S"]))
    assert np.array_equal(Y, np.array(g["Y"]))
    for c in g["cases"]:
        dX, dA, dB, dS = orc.backward(X, W, [A], [B], [g["scale"]], off, np.array(c["dY"]))
        assert np.array_equal(dS[0], np.array(c["dS"]))
        assert np.array_equal(dX, np.array(c["dX"]))
        assert np.array_equal(dA[0], np.array(c["dA"]))
        assert np.array_equal(dB[0], np.array(c["dB"]))


# -- 2. brute force: pure-Python triple loops of the definition -------------------------------------
def _loops(X, W, A, B, scales, off, dY):
    T, d_in = X.shape
    d_out = W.shape[1]
    Y = [[0.0] * d_out for _ in range(T)]
    dX = [[0.0] * d_in for _ in range(T)]
    dA = [[[0.0] * A[j].shape[1] for _ in range(d_in)] for j in range(len(A))]
    dB = [[[0.0] * d_out for _ in range(B[j].shape[0])] for j in range(len(A))]
    for j in range(len(A)):
        r = A[j].shape[1]
        s = scales[j]
        for t in range(off[j], off[j + 1]):
            S = [sum(X[t, i] * A[j][i, p] for i in range(d_in)) for p in range(r)]
            dS = [sum(dY[t, o] * B[j][p, o] for o in range(d_out)) for p in range(r)]
            for o in range(d_out):
                Y[t][o] = sum(X[t, i] * W[i, o] for i in range(d_in)) + s * sum(S[p] * B[j][p, o] for p in range(r))
            for i in range(d_in):
                dX[t][i] = sum(dY[t, o] * W[i, o] for o in range(d_out)) + s * sum(dS[p] * A[j][i, p] for p in range(r))
                for p in range(r):
                    dA[j][i][p] += s * X[t, i] * dS[p]
            for p in range(r):
                for o in range(d_out):
                    dB[j][p][o] += s * S[p] * dY[t, o]
    return np.array(Y), np.array(dX), [np.array(a) for a in dA], [np.array(b) for b in dB]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_loops(seed):
    X, W, A, B, sc, off, dY = _tiny(seed, d_in=6, d_out=4, ranks=(2, 1, 3), tokens=(3, 1, 4), scales=(2.0, 0.5, 3.0))
    Y, dX, dA, dB = _loops(X, W, A, B, sc, off, dY)
    Yo, _ = orc.forward(X, W, A, B, sc, off)
    dXo, dAo, dBo, _ = orc.backward(X, W, A, B, sc, off, dY)
    np.testing.assert_allclose(Yo, Y, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dXo, dX, rtol=1e-13, atol=1e-13)
    for j in range(3):
        np.testing.assert_allclose(dAo[j], dA[j], rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(dBo[j], dB[j], rtol=1e-13, atol=1e-13)


# -- 3. central finite differences of L = sum(dY * Y) ---------------------------------------------------
def test_finite_differences():
    X, W, A, B, sc, off, dY = _tiny(3)
    dX, dA, dB, _ = orc.backward(X, W, A, B, sc, off, dY)
    h = 1e-6

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + h
        lp = orc.loss(X, W, A, B, sc, off, dY)
        arr[idx] = old - h
        lm = orc.loss(X, W, A, B, sc, off, dY)
        arr[idx] = old
        return (lp - lm) / (2 * h)

    for idx in np.ndindex(*X.shape):
        assert abs(fd(X, idx) - dX[idx]) <= 1e-7 * (1 + abs(dX[idx]))
    for j in range(len(A)):
        for idx in np.ndindex(*A[j].shape):
            assert abs(fd(A[j], idx) - dA[j][idx]) <= 1e-7 * (1 + abs(dA[j][idx]))
        for idx in np.ndindex(*B[j].shape):
            assert abs(fd(B[j], idx) - dB[j][idx]) <= 1e-7 * (1 + abs(dB[j][idx]))


# -- 4. B = 0 special case: the layer is the backbone GEMM --------------------------------------------------
def test_zero_B_reduces_to_backbone():
    X, W, A, B, sc, off, dY = _tiny(4, d_in=9, d_out=11, ranks=(2, 4), tokens=(5, 3))
    B0 = [np.zeros_like(b) for b in B]
    Y, S = orc.forward(X, W, A, B0, sc, off)
    assert np.array_equal(Y, X @ W)
    dX, dA, dB, _ = orc.backward(X, W, A, B0, sc, off, dY)
    assert np.array_equal(dX, dY @ W.T)
    assert all(np.all(a == 0) for a in dA)
    assert all(np.any(b != 0) for b in dB)          # dB does not vanish: the adapter still learns
    # and dB_j = s_j (X_j A_j)^T dY_j, checked with einsum rather than matmul
    for j in range(2):
        lo, hi = off[j], off[j + 1]
        ref = sc[j] * np.einsum("ti,ip,to->po", X[lo:hi], A[j], dY[lo:hi])
        np.testing.assert_allclose(dB[j], ref, rtol=1e-12, atol=1e-12)


# -- 5. three-way identity: fused == each job alone == dense X.(W + s A B) -----------------------------------
def test_fused_equals_per_job_equals_dense():
    wl = wk.config(0)
    p = wk.generate(wl)
    off = p.offsets
    Y, _ = orc.forward(p.X, p.W, p.A, p.B, p.scales, off)
    dX, dA, dB, _ = orc.backward(p.X, p.W, p.A, p.B, p.scales, off, p.dY)
    X, W, dY = (np.asarray(a, np.float64) for a in (p.X, p.W, p.dY))
    for j in range(wl.num_jobs):
        lo, hi = int(off[j]), int(off[j + 1])
        Aj, Bj, s = np.asarray(p.A[j], np.float64), np.asarray(p.B[j], np.float64), p.scales[j]
        # the job on its own
        Y1, _ = orc.forward(X[lo:hi], W, [Aj], [Bj], [s], [0, hi - lo])
        dX1, dA1, dB1, _ = orc.backward(X[lo:hi], W, [Aj], [Bj], [s], [0, hi - lo], dY[lo:hi])
        assert np.array_equal(Y[lo:hi], Y1) and np.array_equal(dX[lo:hi], dX1)
        assert np.array_equal(dA[j], dA1[0]) and np.array_equal(dB[j], dB1[0])
        # the dense layer with the merged weight, and its weight gradient pushed through A.B
        Weff = W + s * np.einsum("ip,po->io", Aj, Bj)
        np.testing.assert_allclose(Y[lo:hi], np.einsum("ti,io->to", X[lo:hi], Weff), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dX[lo:hi], np.einsum("to,io->ti", dY[lo:hi], Weff), rtol=1e-12, atol=1e-12)
        dWeff = np.einsum("ti,to->io", X[lo:hi], dY[lo:hi])
        np.testing.assert_allclose(dA[j], s * np.einsum("io,po->ip", dWeff, Bj), rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(dB[j], s * np.einsum("ip,io->po", Aj, dWeff), rtol=1e-11, atol=1e-11)


# -- 6. structural invariants -------------------------------------------------------------------------
def test_identity_input_exposes_merged_weight():
    rng = np.random.default_rng(5)
    d_in, d_out, r = 6, 4, 2
    W, A, B = rng.standard_normal((d_in, d_out)), rng.standard_normal((d_in, r)), rng.standard_normal((r, d_out))
    Y, _ = orc.forward(np.eye(d_in), W, [A], [B], [1.5], [0, d_in])
    ref = W.copy()
    for i in range(d_in):
        for o in range(d_out):
            ref[i, o] += 1.5 * sum(A[i, p] * B[p, o] for p in range(r))
    np.testing.assert_allclose(Y, ref, rtol=1e-14, atol=1e-14)


def test_jobs_are_independent_and_permutable():
    X, W, A, B, sc, off, dY = _tiny(6, d_in=8, d_out=6, ranks=(2, 3, 1), tokens=(4, 2, 3), scales=(1.0, 2.0, 0.5))
    Y, _ = orc.forward(X, W, A, B, sc, off)
    dX, dA, dB, _ = orc.backward(X, W, A, B, sc, off, dY)
    # perturbing job 1 leaves job 0 / job 2 outputs bit-identical
    X2, A2, B2 = X.copy(), [a.copy() for a in A], [b.copy() for b in B]
    X2[off[1]:off[2]] += 1.0
    A2[1] *= 3.0
    B2[1] -= 1.0
    Y2, _ = orc.forward(X2, W, A2, B2, sc, off)
    dX2, dA2, dB2, _ = orc.backward(X2, W, A2, B2, sc, off, dY)
    for j in (0, 2):
        sl = slice(off[j], off[j + 1])
        assert np.array_equal(Y[sl], Y2[sl]) and np.array_equal(dX[sl], dX2[sl])
        assert np.array_equal(dA[j], dA2[j]) and np.array_equal(dB[j], dB2[j])
    # permuting the jobs together with their segments permutes the outputs
    perm = [2, 0, 1]
    segs = [slice(off[j], off[j + 1]) for j in range(3)]
    Xp = np.concatenate([X[segs[j]] for j in perm])
    dYp = np.concatenate([dY[segs[j]] for j in perm])
    offp = np.concatenate([[0], np.cumsum([off[j + 1] - off[j] for j in perm])])
    Yp, _ = orc.forward(Xp, W, [A[j] for j in perm], [B[j] for j in perm], [sc[j] for j in perm], offp)
    dXp, dAp, dBp, _ = orc.backward(Xp, W, [A[j] for j in perm], [B[j] for j in perm], [sc[j] for j in perm], offp, dYp)
    for k, j in enumerate(perm):
        slp = slice(offp[k], offp[k + 1])
        assert np.array_equal(Yp[slp], Y[segs[j]]) and np.array_equal(dXp[slp], dX[segs[j]])
        assert np.array_equal(dAp[k], dA[j]) and np.array_equal(dBp[k], dB[j])


def test_split_segment_adds_gradients_and_scale_is_affine():
    rng = np.random.default_rng(7)
    d_in, d_out, r, T = 7, 5, 3, 6
    X, W, dY = rng.standard_normal((T, d_in)), rng.standard_normal((d_in, d_out)), rng.standard_normal((T, d_out))
    A, B = rng.standard_normal((d_in, r)), rng.standard_normal((r, d_out))
    _, dA1, dB1, _ = orc.backward(X, W, [A], [B], [2.0], [0, T], dY)
    _, dA2, dB2, _ = orc.backward(X, W, [A, A], [B, B], [2.0, 2.0], [0, 2, T], dY)
    np.testing.assert_allclose(dA1[0], dA2[0] + dA2[1], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dB1[0], dB2[0] + dB2[1], rtol=1e-13, atol=1e-13)
    Y0, _ = orc.forward(X, W, [A], [B], [0.0], [0, T])
    Y1, _ = orc.forward(X, W, [A], [B], [1.0], [0, T])
    Y3, _ = orc.forward(X, W, [A], [B], [3.0], [0, T])
    np.testing.assert_allclose(Y3 - Y0, 3.0 * (Y1 - Y0), rtol=1e-12, atol=1e-12)
    assert np.array_equal(Y0, X @ W)


def test_row_sampling_matches_full_and_empty_segments():
    X, W, A, B, sc, off, dY = _tiny(8, d_in=8, d_out=6, ranks=(2, 3, 1), tokens=(4, 0, 3), scales=(1.0, 2.0, 0.5))
    Y, S = orc.forward(X, W, A, B, sc, off)
    dX, dA, dB, dS = orc.backward(X, W, A, B, sc, off, dY)
    assert S[1].shape == (0, 3) and np.all(dA[1] == 0) and np.all(dB[1] == 0)
    rows = np.array([6, 0, 3, 4])
    Ys, _ = orc.forward(X, W, A, B, sc, off, rows=rows)
    dXs, *_ = orc.backward(X, W, A, B, sc, off, dY, rows=rows)
    np.testing.assert_allclose(Ys, Y[rows], rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(dXs, dX[rows], rtol=1e-14, atol=1e-14)
    assert list(orc.job_of_rows(off, rows)) == [2, 0, 0, 2]


def test_rank_zero_job_is_backbone_only():
    rng = np.random.default_rng(9)
    X, W, dY = rng.standard_normal((4, 5)), rng.standard_normal((5, 3)), rng.standard_normal((4, 3))
    A, B = [np.zeros((5, 0))], [np.zeros((0, 3))]
    Y, _ = orc.forward(X, W, A, B, [2.0], [0, 4])
    dX, dA, dB, _ = orc.backward(X, W, A, B, [2.0], [0, 4], dY)
    assert np.array_equal(Y, X @ W) and np.array_equal(dX, dY @ W.T)
    assert dA[0].shape == (5, 0) and dB[0].shape == (0, 3)


# -- integer bookkeeping --------------------------------------------------------------------------------
def test_bookkeeping_closed_forms():
    assert [orc.padded_rank(r) for r in (0, 1, 3, 8, 9, 48, 256)] == [0, 8, 8, 8, 16, 48, 256]
    tiles = orc.row_tiles([0, 3, 3, 300, 520], 256)
    assert tiles == [(0, 256, 0, 2), (256, 256, 2, 3), (512, 8, 3, 3)]


def test_workload_tables_follow_the_stated_recipe():
    c1, c2 = wk.config(1), wk.config(2)
    assert c1.total_tokens == 7680 and list(c1.ranks) == [8, 16, 32, 64]
    assert list(c2.tokens) == [5120, 512, 2048, 3584, 3072, 6144, 5120, 6144] and c2.total_tokens == 31744
    assert abs(c1.flops() - 0.525e12) < 0.002e12
    assert abs(c2.flops() - 19.62e12) < 0.02e12
    c3, c4 = wk.config(3), wk.config(4)
    assert c3.num_jobs == 16 and c3.total_tokens == 83968
    assert c4.num_jobs == 32 and {1, 17, 333, 16384} <= set(c4.tokens)
    assert set(c4.ranks) <= {1, 3, 8, 48, 96, 256} and all(0.5 <= s <= 4.0 for s in c4.scales)
    p = wk.generate(wk.config(0))
    assert p.X.shape == (128, 256) and p.A[1].shape == (256, 8) and p.B[0].shape == (4, 256)
    assert abs(float(p.W.std()) - 0.02) < 1e-3 and abs(float(p.B[1].std()) - 0.01) < 2e-3
    assert float(np.abs(p.A[0]).max()) <= 1 / 16
    # bf16 rounding is round-to-nearest-even on the top 16 bits
    x = np.array([1.0, 1.00390625, 1.01171875, -3.140625, 1e-3], dtype=np.float32)
    r = wk.round_to_bf16(x)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert r[1] == np.float32(1.0) and r[2] == np.float32(1.015625)      # ties go to the even mantissa
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
