"""GPU parity on tensors at and beyond 4 GiB.

1. Contiguous calls: 2.1 million tokens through a 2048 -> 1024 projection, so that X and dX hold 2^32 elements
   (8.6 GB each) and Y and dY 4.3 GB -- element offsets beyond 2^31 and byte offsets beyond 2^33 inside every kernel
   of the path.  Two jobs of about a million tokens (their dA / dB sums run over a million rows), a 77-token job
   between them and a rank-0 job at the end.
2. Token-indexed calls with X just below 4 GiB (1 048 000 tokens x 2048), the largest the kernels read through the
   row list directly: their per-lane byte offsets from the tensor base are 32 bits wide and here come within 2.4 MB of 2^32.
   The rows of the jobs are spread over the batch by a random permutation.

Inputs are drawn on the device with a seeded generator (the workloads' distributions); the fp64 oracle runs chunk by
chunk over ALL rows: every element of Y and dX is compared, dA_j and dB_j are accumulated over the chunks in float64
and compared in full.  For the indexed call the oracle is the contiguous one applied to the rows in job order (the
token-by-token indexed oracle is pinned to exactly that equivalence on the CPU, and is far too slow for 10^6 rows)."""
import numpy as np
import pytest

from oracle import tlora_oracle as orc
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

D_IN, D_OUT = 2048, 1024
CHUNK = 65536


def _run(tag, ranks, tokens, scales, indexed, seed):
    import torch
    from paper_2602_07263_amd import tlora
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    bf = torch.bfloat16
    X = torch.empty(T, D_IN, dtype=bf, device="cuda")
    dY = torch.empty(T, D_OUT, dtype=bf, device="cuda")
    for c0 in range(0, T, 4 * CHUNK):                       # drawn in pieces: no fp32 copy of a whole tensor
        c1 = min(T, c0 + 4 * CHUNK)
        X[c0:c1] = torch.randn(c1 - c0, D_IN, device="cuda", generator=g).to(bf)
        dY[c0:c1] = torch.randn(c1 - c0, D_OUT, device="cuda", generator=g).to(bf)
    W = (torch.randn(D_IN, D_OUT, device="cuda", generator=g) * 0.02).to(bf)
    A = [((torch.rand(D_IN, r, device="cuda", generator=g) * 2 - 1) / D_IN ** 0.5).to(bf) for r in ranks]
    B = [(torch.randn(r, D_OUT, device="cuda", generator=g) * 0.01).to(bf) for r in ranks]
    lp = tlora.LayerProblem("bf16", D_IN, D_OUT, ranks, off, scales, X, W, A, B)
    Y, dX, dA, dB = lp.new_outputs()
    print(f"{tag}: T={T}, X {X.numel() * 2 / 2**30:.2f} GiB, Y {Y.numel() * 2 / 2**30:.2f} GiB: forward + backward", flush=True)
    if indexed:
        index = torch.randperm(T, device="cuda", generator=g).to(torch.int32)      # sorted position -> batch row
        ws_bytes = tlora.tlora_indexed_workspace_bytes(lp.prob)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        st = int(torch.cuda.current_stream().cuda_stream)
        ptrs = lambda ts: [t.data_ptr() if t.numel() else 0 for t in ts]
        tlora.tlora_fwd_indexed(lp.prob, index.data_ptr(), Y.data_ptr(), ws.data_ptr(), ws_bytes, st)
        tlora.tlora_bwd_indexed(lp.prob, index.data_ptr(), dY.data_ptr(), dX.data_ptr(), ptrs(dA), ptrs(dB),
                                tlora.TLORA_BWD_REUSE_S, ws.data_ptr(), ws_bytes, st)
        rows_of = lambda c0, c1: index[c0:c1].long()
    else:
        lp.fwd(Y)
        lp.bwd(dY, dX, dA, dB, reuse_S=True)
        rows_of = lambda c0, c1: slice(c0, c1)
    torch.cuda.synchronize()
    print(f"{tag}: GPU done; oracle over all rows, chunk by chunk", flush=True)

    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    Wh, Ah, Bh = host(W), [host(a) for a in A], [host(b) for b in B]
    dA_ref = [np.zeros((D_IN, r)) for r in ranks]
    dB_ref = [np.zeros((r, D_OUT)) for r in ranks]
    worst = {"Y": 0.0, "dX": 0.0}
    for n, c0 in enumerate(range(0, T, CHUNK)):
        c1 = min(T, c0 + CHUNK)
        loc = np.clip(off, c0, c1) - c0                      # the jobs' segments inside this chunk of the job order
        rows = rows_of(c0, c1)
        Yr, _S = orc.forward(host(X[rows]), Wh, Ah, Bh, scales, loc)
        dXr, dAr, dBr, _dS = orc.backward(host(X[rows]), Wh, Ah, Bh, scales, loc, host(dY[rows]))
        worst["Y"] = max(worst["Y"], pu.worst_ratio(host(Y[rows]), Yr, pu.BF16_TOL))
        worst["dX"] = max(worst["dX"], pu.worst_ratio(host(dX[rows]), dXr, pu.BF16_TOL))
        for j in range(len(ranks)):
            dA_ref[j] += dAr[j]
            dB_ref[j] += dBr[j]
        if n % 8 == 7:
            print(f"{tag}: {c1} rows checked, worst ratios so far {worst}", flush=True)
    worst["dA"] = max(pu.worst_ratio(a.cpu().numpy(), r, pu.BF16_TOL) for a, r in zip(dA, dA_ref))
    worst["dB"] = max(pu.worst_ratio(b.cpu().numpy(), r, pu.BF16_TOL) for b, r in zip(dB, dB_ref))
    print(f"{tag}: worst error / tolerance ratios {worst}", flush=True)
    bad = {k: v for k, v in worst.items() if not v <= 1.0}
    assert not bad, f"{tag}: worst error / tolerance ratios {worst}"


def test_fused_layer_on_tensors_beyond_four_gib():
    tokens = [1_100_000, 77, 997_075, 333]
    assert sum(tokens) * D_IN >= 2 ** 32 and sum(tokens) * D_OUT * 2 >= 2 ** 32
    _run("large offsets", [8, 64, 3, 0], tokens, [2.0, 0.5, 1.5, 1.0], indexed=False, seed=4242)


def test_indexed_calls_with_row_offsets_up_to_four_gib():
    tokens = [500_000, 123, 547_877]
    T = sum(tokens)
    assert 2 ** 32 - 2 ** 23 <= T * D_IN * 2 < 2 ** 32           # the direct path's bound, nearly reached
    _run("indexed, 32-bit row offsets", [16, 130, 5], tokens, [2.0, 0.5, 1.5], indexed=True, seed=4343)
