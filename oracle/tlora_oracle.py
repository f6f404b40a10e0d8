"""fp64 CPU oracle for the fused multi-LoRA linear layer.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's `cpu_baseline` leg may import this
module; the product path never does.  It shares no code with the HIP implementation and
imports nothing but numpy.

What it computes is the plain definition of the layer, one job at a time, in float64:

  forward   (Sec. 3.3, fused batched LoRA kernel: tokens of adapter i are multiplied by the
             down-projection A_i into a compact |X_i| x r_i intermediate, which is multiplied by
             the up-projection B_i and added to the shared-backbone product; Sec. 2: W + dW with
             dW = A.B, A: d x r, B: r x k -- the paper prints a transpose on B that its own
             shapes rule out):
      S_j   = X_j . A_j
      Y_j   = X_j . W + scale_j * S_j . B_j
  backward  (Sec. 3.2: every job keeps independent forward/backward semantics and the backbone W
             is frozen; the paper gives no formulas, these are the derivatives of
             L = sum(dY * Y) ):
      dS_j  = dY_j . B_j^T
      dX_j  = dY_j . W^T + scale_j * dS_j . A_j^T
      dA_j  = scale_j * X_j^T . dS_j
      dB_j  = scale_j * S_j^T . dY_j
      (no dW)

`X_j` is the contiguous row block offsets[j]:offsets[j+1].  Each product is one numpy float64
matmul (a library primitive used as a single step); there is no blocking, fusion or reordering.
`rows` restricts Y / dX to a subset of token rows (each row of Y and dX depends only on its
own row of X / dY and on its job's adapter), so large problems can be checked on samples.

Every function here is pinned by tests/test_oracle_pins.py against values that do not come
from this file: a hand-worked 2x2 example, pure-Python triple loops, central finite
differences, the dense-weight identity X.(W + s.A.B), the B = 0 special case and structural
invariants.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def job_of_rows(offsets: Sequence[int], rows: np.ndarray) -> np.ndarray:
    """Index of the job whose segment holds each row (empty segments own no row)."""
    off = np.asarray(offsets, dtype=np.int64)
    return np.searchsorted(off, np.asarray(rows, dtype=np.int64), side="right") - 1


def shrink(X, A: Sequence, offsets) -> List[np.ndarray]:
    """S_j = X_j . A_j  for every job (the compact |X_j| x r_j intermediates of Sec. 3.3)."""
    X = _f64(X)
    return [X[offsets[j]:offsets[j + 1]] @ _f64(A[j]) for j in range(len(A))]


def forward(X, W, A: Sequence, B: Sequence, scales, offsets,
            rows: Optional[np.ndarray] = None) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Y (all rows, or the given rows in the given order) and the full S_j list."""
    X, W = _f64(X), _f64(W)
    J = len(A)
    S = shrink(X, A, offsets)
    if rows is None:
        Y = np.empty((X.shape[0], W.shape[1]), dtype=np.float64)
        for j in range(J):
            lo, hi = int(offsets[j]), int(offsets[j + 1])
            Y[lo:hi] = X[lo:hi] @ W + float(scales[j]) * (S[j] @ _f64(B[j]))
        return Y, S
    rows = np.asarray(rows, dtype=np.int64)
    jobs = job_of_rows(offsets, rows)
    Y = X[rows] @ W
    for j in range(J):
        sel = np.nonzero(jobs == j)[0]
        if sel.size:
            local = rows[sel] - int(offsets[j])
            Y[sel] += float(scales[j]) * (S[j][local] @ _f64(B[j]))
    return Y, S


def backward(X, W, A: Sequence, B: Sequence, scales, offsets, dY,
             rows: Optional[np.ndarray] = None):
    """(dX, dA list, dB list, dS list).  dX covers all rows or the given rows."""
    X, W, dY = _f64(X), _f64(W), _f64(dY)
    J = len(A)
    S = shrink(X, A, offsets)
    dS, dA, dB = [], [], []
    for j in range(J):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        s = float(scales[j])
        dS_j = dY[lo:hi] @ _f64(B[j]).T
        dS.append(dS_j)
        dA.append(s * (X[lo:hi].T @ dS_j))
        dB.append(s * (S[j].T @ dY[lo:hi]))
    if rows is None:
        dX = np.empty_like(X)
        for j in range(J):
            lo, hi = int(offsets[j]), int(offsets[j + 1])
            dX[lo:hi] = dY[lo:hi] @ W.T + float(scales[j]) * (dS[j] @ _f64(A[j]).T)
    else:
        rows = np.asarray(rows, dtype=np.int64)
        jobs = job_of_rows(offsets, rows)
        dX = dY[rows] @ W.T
        for j in range(J):
            sel = np.nonzero(jobs == j)[0]
            if sel.size:
                local = rows[sel] - int(offsets[j])
                dX[sel] += float(scales[j]) * (dS[j][local] @ _f64(A[j]).T)
    return dX, dA, dB, dS


def loss(X, W, A, B, scales, offsets, dY) -> float:
    """L = sum(dY * Y): the scalar whose derivatives `backward` returns."""
    Y, _ = forward(X, W, A, B, scales, offsets)
    return float(np.sum(_f64(dY) * Y))


# ---- integer bookkeeping (bit-exact side of the parity bar) --------------------------------------

def padded_rank(r: int, granule: int = 8) -> int:
    """Rank rounded up to the padding granule (0 stays 0)."""
    return (int(r) + granule - 1) // granule * granule


def row_tiles(offsets: Sequence[int], tile_rows: int) -> List[Tuple[int, int, int, int]]:
    """Uniform row tiles over the concatenated batch: (row0, rows, first_job, last_job), where
    first/last are the first and last jobs with at least one row inside the tile."""
    T = int(offsets[-1])
    tiles = []
    for row0 in range(0, T, tile_rows):
        rows = min(tile_rows, T - row0)
        present = [j for j in range(len(offsets) - 1)
                   if int(offsets[j]) < row0 + rows and int(offsets[j + 1]) > row0]
        tiles.append((row0, rows, present[0], present[-1]))
    return tiles
