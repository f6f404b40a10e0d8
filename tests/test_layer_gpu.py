"""GPU parity of one whole decoder layer (attention half, then MLP half; seven fused multi-LoRA projections) against
the fp64 oracle on the same seeded bf16 inputs; the oracle rounds the tensors the layer keeps in memory between its
kernels at the same points."""
import numpy as np
import pytest

from oracle import layer_oracle as ly
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
HD = 128


def test_decoder_layer_matches_oracle():
    import torch
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv = 256, 640, 4, 2
    ranks, tokens, scales = [8, 0, 24, 3], [300, 0, 513, 70], [2.0, 1.0, 0.5, 4.0]
    seq = np.array([0, 100, 300, 301, 600, 813, 883], dtype=np.int64)
    eps, base = 1e-5, 10000.0
    rng = np.random.default_rng(8)
    f = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32))
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    layers = {n: (f(rng.normal(size=(i, o)) / np.sqrt(i)), [f(rng.uniform(-1, 1, size=(i, r)) / np.sqrt(i)) for r in ranks],
                  [f(0.05 * rng.normal(size=(r, o))) for r in ranks]) for n, (i, o) in shapes.items()}
    X, dOut = f(rng.normal(size=(T, d))), f(rng.normal(size=(T, d)))
    g_attn, g_mlp = f(1.0 + 0.1 * rng.normal(size=d)), f(1.0 + 0.1 * rng.normal(size=d))
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, base, ranks, off, scales, seq, up(X), up(g_attn), up(g_mlp), eps, tl)
    Out = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dX = torch.full_like(Out, float("nan"))
    grads = layer.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    layer.fwd(Out)
    layer.bwd(up(dOut), dX, grads)
    torch.cuda.synchronize()
    store = lambda a: wk.round_to_bf16(a.astype(np.float32)).astype(np.float64)
    attn = (g_attn, eps, {n: layers[n] for n in ("q", "k", "v", "o")})
    mlp = (g_mlp, eps, {n: layers[n] for n in ("gate", "up", "down")})
    args = (attn, mlp, scales, off, seq, Hq, Hkv, HD, base)
    out_r, _ = ly.forward(X, *args, store)
    dX_r, g_r = ly.backward(X, *args, dOut, store)
    # two blocks chained: each block's error budget (see the block tests) adds
    tol = 2 * pu.BF16_TOL

    def ratio(got, ref):
        # |err| <= tol (m + |ref|), m = max(1, rms(ref)): gradients that are long sums of products of bf16-stored
        # tensors carry one-ulp flips of those as noise relative to the sum's typical size
        if ref.size == 0:
            return 0.0
        got = np.asarray(got, dtype=np.float64)
        assert np.all(np.isfinite(got))
        m = max(1.0, float(np.sqrt(np.mean(ref * ref))))
        return float(np.max(np.abs(got - ref) / (tol * (m + np.abs(ref)))))
    res = {"Out": ratio(Out.float().cpu().numpy(), out_r), "dX": ratio(dX.float().cpu().numpy(), dX_r)}
    for n in grads:
        res["dA_" + n] = max([ratio(a.cpu().numpy(), r) for a, r in zip(grads[n][0], g_r[n][0])] + [0.0])
        res["dB_" + n] = max([ratio(b.cpu().numpy(), r) for b, r in zip(grads[n][1], g_r[n][1])] + [0.0])
    print({k: round(v, 3) for k, v in res.items()})
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {res}"


def test_decoder_layer_without_tokens_gives_zero_gradients():
    import torch
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv = 256, 384, 2, 1
    ranks = [4, 8]
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    rn = lambda *sh: torch.randn(*sh, device="cuda", generator=g).to(torch.bfloat16)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    tl = {n: (rn(i, o), [rn(i, r) for r in ranks], [rn(r, o) for r in ranks]) for n, (i, o) in shapes.items()}
    X = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    gamma = torch.ones(d, dtype=torch.bfloat16, device="cuda")
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, 10000.0, ranks, [0, 0, 0], [1.0, 2.0], [0], X, gamma, gamma, 1e-5, tl)
    grads = layer.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    layer.fwd(X)
    layer.bwd(X, X, grads)
    torch.cuda.synchronize()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            assert float(t.abs().max()) == 0.0, n
