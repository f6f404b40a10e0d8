"""GPU parity of the MLP block (RMSNorm -> gate / up -> gated SiLU -> down -> residual over fused multi-LoRA
projections) against the fp64 oracle on the same seeded inputs.  The results must hold the tolerance against the plain fp64
oracle and against the oracle that rounds the tensors the block keeps in memory between its kernels."""
import numpy as np
import pytest

from oracle import mlp_oracle as mo
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _make(dtype, d, dff, ranks, tokens, scales, seed):
    rng = np.random.default_rng(seed)
    rnd = wk.round_to_bf16 if dtype == "bf16" else (lambda a: a)
    f = lambda a: rnd(np.asarray(a, dtype=np.float32))
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    X = f(rng.normal(size=(T, d)))
    gamma = f(1.0 + 0.1 * rng.normal(size=d))
    layers = {}
    for name, (i, o) in dict(gate=(d, dff), up=(d, dff), down=(dff, d)).items():
        W = f(rng.normal(size=(i, o)) / np.sqrt(i))
        A = [f(rng.uniform(-1, 1, size=(i, r)) / np.sqrt(i)) for r in ranks]
        B = [f(0.05 * rng.normal(size=(r, o))) for r in ranks]
        layers[name] = (W, A, B)
    dOut = f(rng.normal(size=(T, d)))
    return X, gamma, layers, off, dOut


CASES = [("bf16", 256, 640, [8, 0, 24, 3], [300, 0, 513, 70], [2.0, 1.0, 0.5, 4.0]),
         ("f32", 64, 96, [4, 7], [50, 81], [2.0, 1.0]),
         ("bf16", 128, 384, [1, 130], [129, 260], [1.5, 1.5]),
         ("bf16", 512, 1024, [32], [515], [1.0]),
         ("bf16", 384, 200, [5, 0, 16], [64, 200, 7], [1.0, 1.0, 3.0])]


@pytest.mark.parametrize("case", CASES, ids=["bf16", "f32", "bf16_odd_ranks", "bf16_one_job", "bf16_narrow_ff"])
def test_mlp_block_matches_oracle(case):
    import torch
    from paper_2602_07263_amd import tlora
    dtype, d, dff, ranks, tokens, scales = case
    X, gamma, layers, off, dOut = _make(dtype, d, dff, ranks, tokens, scales, seed=4)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=tdt).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    blk = tlora.MlpBlock(dtype, d, dff, ranks, off, scales, up(X), up(gamma), 1e-5, tl)
    Out = torch.full((sum(tokens), d), float("nan"), dtype=tdt, device="cuda")
    dX = torch.full_like(Out, float("nan"))
    grads = blk.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    blk.fwd(Out)
    blk.bwd(up(dOut), dX, grads)
    torch.cuda.synchronize()
    # bf16: every path crosses two fused layers (gate / up, then down), each with the layer's budget: the budgets add
    # (measured against one budget: 0.25 - 1.0 over the shapes above).  fp32: chained fp32 layers and glue stages.
    # Out and dX have rms ~ 1 and are held to tol (1 + |ref|); the adapter gradients to tol (max(1, rms) + |ref|).
    tol = 2 * pu.BF16_TOL if dtype == "bf16" else 2e-5

    def oracle(store):
        out_r, _ = mo.forward(X, gamma, 1e-5, layers, scales, off, store)
        dX_r, g_r = mo.backward(X, gamma, 1e-5, layers, scales, off, dOut, store)
        return out_r, dX_r, g_r
    res = pu.block_report(f"MLP block {dtype}", Out, dX, grads, oracle, tol, pu.bf16_store if dtype == "bf16" else (lambda a: a))
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"{dtype}: worst error / tolerance ratios {res}"
