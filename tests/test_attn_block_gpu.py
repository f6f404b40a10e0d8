"""GPU parity of the attention block (RMSNorm -> q / k / v fused multi-LoRA projections -> rotary embedding -> causal
grouped-query attention -> o projection -> residual) against the fp64 oracle on the same seeded bf16 inputs.  The results must hold the
tolerance against the plain fp64 oracle and against the oracle that rounds the tensors the block keeps in memory
between its kernels."""
import numpy as np
import pytest

from oracle import attn_oracle as ao
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
HD = 128
# Every path through the block crosses two fused layers (q / k / v, then o), each with the layer's error budget, and an
# attention between them whose matrix units take bf16 probabilities and score gradients: the budgets add.  (Measured:
# the worst ratio against one budget lies between 0.7 and 1.2 over the shapes below; the float64 run of the oracle
# against itself with the stored tensors disturbed by a few fp32 ulps -- rounding flips alone -- in
# tests/test_tolerance_derivations.py gives 0.1 to 0.8 of one budget.)  Adapter gradients are held to
# tol (max(1, rms(ref)) + |ref|), see parity_util.rms_floor_ratio.
BLOCK_TOL = 2 * pu.BF16_TOL


def _make(d, Hq, Hkv, ranks, tokens, seed):
    rng = np.random.default_rng(seed)
    f = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32))
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    X = f(rng.normal(size=(T, d)))
    gamma = f(1.0 + 0.1 * rng.normal(size=d))
    layers = {}
    for name, (i, o) in dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d)).items():
        W = f(rng.normal(size=(i, o)) / np.sqrt(i))
        A = [f(rng.uniform(-1, 1, size=(i, r)) / np.sqrt(i)) for r in ranks]
        B = [f(0.05 * rng.normal(size=(r, o))) for r in ranks]
        layers[name] = (W, A, B)
    dOut = f(rng.normal(size=(T, d)))
    return X, gamma, layers, off, dOut


def test_attn_block_matches_oracle():
    import torch
    from paper_2602_07263_amd import tlora
    d, Hq, Hkv = 256, 4, 2
    ranks, tokens, scales = [8, 0, 24, 3], [300, 0, 513, 70], [2.0, 1.0, 0.5, 4.0]
    # every job's tokens are whole sequences: 100 + 200 | - | 1 + 299 + 213 | 70
    seq = np.array([0, 100, 300, 301, 600, 813, 883], dtype=np.int64)
    eps, base = 1e-5, 10000.0
    X, gamma, layers, off, dOut = _make(d, Hq, Hkv, ranks, tokens, seed=6)
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    blk = tlora.AttnBlock(d, Hq, Hkv, base, ranks, off, scales, seq, up(X), up(gamma), eps, tl)
    Out = torch.full((sum(tokens), d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dX = torch.full_like(Out, float("nan"))
    grads = blk.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    blk.fwd(Out)
    blk.bwd(up(dOut), dX, grads)
    torch.cuda.synchronize()
    args = (gamma, eps, layers, scales, off, seq, Hq, Hkv, HD, base)

    def oracle(store):
        out_r, _ = ao.block_forward(X, *args, store)
        dX_r, g_r = ao.block_backward(X, *args, dOut, store)
        return out_r, dX_r, g_r
    res = pu.block_report("attention block", Out, dX, grads, oracle, BLOCK_TOL, pu.bf16_store)
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {res}"


def test_attn_block_rejects_fp32_and_mismatched_sequences():
    import ctypes
    import torch
    from paper_2602_07263_amd import tlora
    d, Hq, Hkv = 256, 2, 1
    X, gamma, layers, off, _ = _make(d, Hq, Hkv, [4], [64], seed=1)
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    with pytest.raises(tlora.TloraError):       # sequences cover 60 tokens, jobs 64
        tlora.AttnBlock(d, Hq, Hkv, 10000.0, [4], off, [1.0], [0, 60], up(X), up(gamma), 1e-5, tl)
    blk = tlora.AttnBlock(d, Hq, Hkv, 10000.0, [4], off, [1.0], [0, 64], up(X), up(gamma), 1e-5, tl)
    blk.prob.dtype = tlora.TLORA_F32
    assert tlora.lib().tlora_attn_workspace_bytes(ctypes.byref(blk.prob)) == 0


def test_attn_block_gradient_accumulation():
    """TLORA_BWD_ACCUMULATE adds to the adapter gradients: a second backward with the flag doubles them (dX is
    overwritten, so it stays the same)."""
    import torch
    from paper_2602_07263_amd import tlora
    d, Hq, Hkv = 256, 2, 1
    ranks, tokens = [8, 3], [130, 70]
    X, gamma, layers, off, dOut = _make(d, Hq, Hkv, ranks, tokens, seed=9)
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    blk = tlora.AttnBlock(d, Hq, Hkv, 10000.0, ranks, off, [1.0, 2.0], [0, 130, 200], up(X), up(gamma), 1e-5, tl)
    Out = torch.empty((200, d), dtype=torch.bfloat16, device="cuda")
    dX1, dX2 = torch.empty_like(Out), torch.empty_like(Out)
    grads = blk.new_grads()
    blk.fwd(Out)
    blk.bwd(up(dOut), dX1, grads)
    torch.cuda.synchronize()
    once = {n: ([a.clone() for a in grads[n][0]], [b.clone() for b in grads[n][1]]) for n in grads}
    blk.bwd(up(dOut), dX2, grads, flags=tlora.TLORA_BWD_ACCUMULATE)
    torch.cuda.synchronize()
    assert torch.equal(dX1.view(torch.int16), dX2.view(torch.int16))
    for n in grads:
        for k in (0, 1):
            for a, b in zip(once[n][k], grads[n][k]):
                assert torch.equal(b, 2 * a), n


@pytest.mark.parametrize("cfg", [(128, 2, 2, [1, 130], [129, 260], [0, 129, 130, 389]),
                                 (384, 3, 1, [5, 0, 16], [64, 200, 7], [0, 64, 164, 264, 271]),
                                 (512, 8, 2, [32], [515], [0, 515])],
                         ids=["odd_ranks", "mqa_rank0_job", "one_job_long_seq"])
def test_attn_block_other_shapes(cfg):
    """Other model widths, head groupings (multi-head, multi-query, grouped), odd ranks (1, 130: two rank blocks),
    a job without adapter, sequences that end off the tile edges."""
    import torch
    from paper_2602_07263_amd import tlora
    d, Hq, Hkv, ranks, tokens, seq = cfg
    scales = [1.5] * len(ranks)
    eps, base = 1e-5, 10000.0
    X, gamma, layers, off, dOut = _make(d, Hq, Hkv, ranks, tokens, seed=17)
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    blk = tlora.AttnBlock(d, Hq, Hkv, base, ranks, off, scales, seq, up(X), up(gamma), eps, tl)
    Out = torch.full((sum(tokens), d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dX = torch.full_like(Out, float("nan"))
    grads = blk.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    blk.fwd(Out)
    blk.bwd(up(dOut), dX, grads)
    torch.cuda.synchronize()
    args = (gamma, eps, layers, scales, off, np.asarray(seq, dtype=np.int64), Hq, Hkv, HD, base)

    def oracle(store):
        out_r, _ = ao.block_forward(X, *args, store)
        dX_r, g_r = ao.block_backward(X, *args, dOut, store)
        return out_r, dX_r, g_r
    res = pu.block_report("attention block", Out, dX, grads, oracle, BLOCK_TOL, pu.bf16_store)
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {res}"
