"""GPU parity on tensors beyond 4 GiB: 2.1 million tokens through a 2048 -> 1024 projection, so that X and dX hold
2^32 elements (8.6 GB each) and Y and dY 4.3 GB -- element offsets beyond 2^31 and byte offsets beyond 2^33 inside
every kernel of the path.  Two jobs of about a million tokens (their dA / dB sums run over a million rows), a
77-token job between them and a rank-0 job at the end.  Inputs are drawn on the device with a seeded generator
(the workloads' distributions); the fp64 oracle runs chunk by chunk over ALL rows: every element of Y and dX is
compared, dA_j and dB_j are accumulated over the chunks in float64 and compared in full."""
import numpy as np
import pytest

from oracle import tlora_oracle as orc
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

D_IN, D_OUT = 2048, 1024
RANKS = [8, 64, 3, 0]
TOKENS = [1_100_000, 77, 997_075, 333]
SCALES = [2.0, 0.5, 1.5, 1.0]
CHUNK = 65536


def test_fused_layer_on_tensors_beyond_four_gib():
    import torch
    from paper_2602_07263_amd import tlora
    T = sum(TOKENS)
    assert T * D_IN >= 2 ** 32 and T * D_OUT * 2 >= 2 ** 32
    off = np.concatenate([[0], np.cumsum(TOKENS)]).astype(np.int64)
    g = torch.Generator(device="cuda")
    g.manual_seed(4242)
    bf = torch.bfloat16
    X = torch.empty(T, D_IN, dtype=bf, device="cuda")
    dY = torch.empty(T, D_OUT, dtype=bf, device="cuda")
    for c0 in range(0, T, 4 * CHUNK):                       # drawn in pieces: no fp32 copy of a whole tensor
        c1 = min(T, c0 + 4 * CHUNK)
        X[c0:c1] = torch.randn(c1 - c0, D_IN, device="cuda", generator=g).to(bf)
        dY[c0:c1] = torch.randn(c1 - c0, D_OUT, device="cuda", generator=g).to(bf)
    W = (torch.randn(D_IN, D_OUT, device="cuda", generator=g) * 0.02).to(bf)
    A = [((torch.rand(D_IN, r, device="cuda", generator=g) * 2 - 1) / D_IN ** 0.5).to(bf) for r in RANKS]
    B = [(torch.randn(r, D_OUT, device="cuda", generator=g) * 0.01).to(bf) for r in RANKS]
    lp = tlora.LayerProblem("bf16", D_IN, D_OUT, RANKS, off, SCALES, X, W, A, B)
    Y, dX, dA, dB = lp.new_outputs()
    print(f"large offsets: T={T}, X {X.numel() * 2 / 2**30:.1f} GiB, Y {Y.numel() * 2 / 2**30:.1f} GiB, "
          f"workspace {lp.ws_bytes / 2**30:.2f} GiB: forward + backward", flush=True)
    lp.fwd(Y)
    lp.bwd(dY, dX, dA, dB, reuse_S=True)
    torch.cuda.synchronize()
    print("large offsets: GPU done; oracle over all rows, chunk by chunk", flush=True)

    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    Wh, Ah, Bh = host(W), [host(a) for a in A], [host(b) for b in B]
    dA_ref = [np.zeros((D_IN, r)) for r in RANKS]
    dB_ref = [np.zeros((r, D_OUT)) for r in RANKS]
    worst = {"Y": 0.0, "dX": 0.0}
    for n, c0 in enumerate(range(0, T, CHUNK)):
        c1 = min(T, c0 + CHUNK)
        loc = np.clip(off, c0, c1) - c0                      # the jobs' segments inside this chunk
        Xc, dYc = host(X[c0:c1]), host(dY[c0:c1])
        Yr, _S = orc.forward(Xc, Wh, Ah, Bh, SCALES, loc)
        dXr, dAr, dBr, _dS = orc.backward(Xc, Wh, Ah, Bh, SCALES, loc, dYc)
        worst["Y"] = max(worst["Y"], pu.worst_ratio(host(Y[c0:c1]), Yr, pu.BF16_TOL))
        worst["dX"] = max(worst["dX"], pu.worst_ratio(host(dX[c0:c1]), dXr, pu.BF16_TOL))
        for j in range(len(RANKS)):
            dA_ref[j] += dAr[j]
            dB_ref[j] += dBr[j]
        if n % 8 == 7:
            print(f"large offsets: rows < {c1} checked, worst ratios so far {worst}", flush=True)
    worst["dA"] = max(pu.worst_ratio(a.cpu().numpy(), r, pu.BF16_TOL) for a, r in zip(dA, dA_ref))
    worst["dB"] = max(pu.worst_ratio(b.cpu().numpy(), r, pu.BF16_TOL) for b, r in zip(dB, dB_ref))
    print(f"large offsets: worst error / tolerance ratios {worst}", flush=True)
    bad = {k: v for k, v in worst.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {worst}"
