"""fp64 CPU oracle of the fused layer with a general token -> adapter assignment.  TEST INFRASTRUCTURE ONLY.

Sec. 3.3 describes the kernel as gathering the tokens of adapter i, multiplying them by A_i and B_i, and
scattering the result back to the output tensor.  The interface: the batch X [T, d_in] is in arbitrary token order;
`row_index` lists the rows job by job (row_index[offsets[j] : offsets[j+1]] are the rows of job j, in the order in
which they enter that job's sums).  Row t of Y / dX belongs to row t of X / dY; dA_j, dB_j sum over the job's rows.
Defined token by token, straight from the layer's formulas (no sorting):

    Y[t]  = X[t].W + s_j (X[t].A_j).B_j                      j = job of row t
    dX[t] = dY[t].W^T + s_j (dY[t].B_j^T).A_j^T
    dA_j  = s_j sum_{t in job j} X[t]^T (dY[t].B_j^T),   dB_j = s_j sum_{t in job j} (X[t].A_j)^T dY[t]

Pinned by tests/test_indexed_pins.py against the contiguous oracle on an explicitly permuted batch and against the
identity permutation.
"""
from __future__ import annotations

import numpy as np


def forward_backward(X, W, A, B, scales, offsets, row_index, dY):
    X, W, dY = (np.asarray(a, dtype=np.float64) for a in (X, W, dY))
    T = X.shape[0]
    Y = np.zeros((T, W.shape[1]))
    dX = np.zeros_like(X)
    dA = [np.zeros(np.asarray(a).shape) for a in A]
    dB = [np.zeros(np.asarray(b).shape) for b in B]
    for j in range(len(A)):
        Aj, Bj, s = np.asarray(A[j], dtype=np.float64), np.asarray(B[j], dtype=np.float64), float(scales[j])
        for pos in range(int(offsets[j]), int(offsets[j + 1])):
            t = int(row_index[pos])
            S = X[t] @ Aj
            Y[t] = X[t] @ W + s * (S @ Bj)
            dS = dY[t] @ Bj.T
            dX[t] = dY[t] @ W.T + s * (dS @ Aj.T)
            dA[j] += s * np.outer(X[t], dS)
            dB[j] += s * np.outer(S, dY[t])
    return Y, dX, dA, dB
